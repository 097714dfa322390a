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
//     are merged through LDS into the range's partial result: normalised values and the
//     log-sum-exp.  A single stream's key ranges are merged INSIDE the same launch, with
//     no fence and no counter: a workgroup publishes its partial result as 64-bit words
//     {fp32 value, 32-bit launch tag} with relaxed device-scope atomic stores, and the
//     workgroups of a kv head share out the result, each reading the words of all ranges
//     with relaxed device-scope atomic loads until every word carries this launch's tag
//     (see merge_ranges; the tag lives in device memory, next to the words).  (A merge
//     by the last workgroup to arrive needs device-scope release/acquire fences, about
//     3 us each here; a second launch costs its gap and a round trip of its own.)  A
//     batch's key ranges are merged by a second, small launch.

#include <hip/hip_bf16.h>

#include <algorithm>
#include <type_traits>

#include "sv_internal.h"

// Measurement build (-DSV_TIMELINE, libsv_timeline.so): the decode kernel stamps the 100 MHz real-time counter at
// a few points into a buffer set with sv_timeline_set, so that one decode step can be laid out on a common clock
// (dispatch, first memory round trip, tile work, merge through LDS and publishing, the reads of the other ranges'
// words, the output's stores), and counts the read attempts of the in-launch merge.  The product build compiles
// none of it.
#ifdef SV_TIMELINE
static __device__ unsigned long long* g_ts = nullptr;   // [8 launch slots][2 kernels][1024 workgroups][8]
#define SV_TS_PARAM , int ts_slot
#define SV_TS_ARG(x) , x
#define SV_TS(kind, wg, i)                                                                                     \
  do {                                                                                                         \
    if (g_ts != nullptr && threadIdx.x == 0 && (wg) < 1024)                                                    \
      g_ts[((((size_t)ts_slot * 2 + (kind)) * 1024 + (wg)) << 3) + (i)] = __builtin_amdgcn_s_memrealtime();     \
  } while (0)
#define SV_TS_VAL(wg, i, v)                                                                                   \
  do {                                                                                                         \
    if (g_ts != nullptr && threadIdx.x == 0 && (wg) < 1024)                                                    \
      g_ts[((((size_t)ts_slot * 2) * 1024 + (wg)) << 3) + (i)] = (v);                                          \
  } while (0)
#define SV_TS_COUNT(v) ++(v)
#else
#define SV_TS_PARAM
#define SV_TS_ARG(x)
#define SV_TS_VAL(wg, i, v) \
  do {                      \
  } while (0)
#define SV_TS_COUNT(v) \
  do {                 \
  } while (0)
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
constexpr int PW = D + 1;      // words a key range publishes per query head: 128 values and the log-sum-exp
// 64-bit header words in front of a tagged region: one per kv head, rounded up to 32
__host__ __device__ static inline int hdr_words_of(int n_kv_heads) { return (n_kv_heads + 31) / 32 * 32; }
constexpr int kPollLimit = 1 << 16;   // polls of a merge read before giving up (each is a memory round trip)

struct DecRow {
  __hip_bfloat16* k;         // K of the layer: kv head 0, slot 0 (written only at the slot of a fused new token)
  __hip_bfloat16* v;
  const float2* cs;          // cos/sin of the query token's rotary angles, [64]
  int32_t len;               // visible keys: slots [0, len), the query token is slot len - 1
  int32_t kps;               // keys per key range of this row (a multiple of 128); ranges = ceil(len / kps)
  int32_t pair0;             // index of the row's first key range among all (row, key range) pairs of the launch
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

// 16 bytes of K or V for launches that read far more than the caches hold (many long streams), every byte once:
// a non-temporal load keeps the stream from displacing itself through L2 and the Infinity Cache (measured
// 16 x 32k tokens: 5.7 -> 6.4 TB/s with merge).  A single stream's 11 MB per layer are partly still cached from
// the step before, and there the plain load is the faster one (10.3 vs 10.9 us per layer-step).
__device__ __forceinline__ uint4 stream_load(const __hip_bfloat16* p) {
  typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

// Rotate, in place, the two 16-byte chunks a lane holds of one row: `lo` covers
// dims [i0, i0 + 8), `hi` the partner dims [i0 + 64, i0 + 72); c/s are cos/sin of
// the 8 pairs.  Result is rounded to bf16, as it would be stored.
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

// ---------------------------------------------------------------------------------
// Merge of the key ranges of one (row, kv head): outputs [o_lo, o_lo + n_out) of its G x 128 (n_out a multiple of 32),
// by one workgroup of NT threads laid out as RG range groups x OPP outputs (RG = 8, 4, 2, 1 for up to 32, 64, 128,
// more outputs): thread (rg, ol) reads output ol from the ranges rg, rg + RG, ... (whole passes of 8, then one pass
// of exactly what is left; all loads of a pass issued before any is looked at) and the RG partial merges meet in
// LDS (3 NT floats at `lds`): one memory round trip unless a thread has more than 8 ranges or the workgroup more
// than NT outputs.
// phk: the partial result of range 0, first query head of the kv head; range s adds s * sstride words, head g adds
// g * PW words.  Words are plain floats, or (POLL) 64-bit {float, launch tag}.
// POLL: the ranges are being written by other workgroups of the SAME launch.  Every word is read with a relaxed
// device-scope atomic load, again and again until it carries this launch's tag: its writer, a workgroup that waits
// for nothing, has then written it, and the value in the same word is the one that goes with it (a 64-bit access is
// single-copy atomic, a word is written once per launch); no ordering between locations is needed.  Workgroups are
// dispatched in index order and the ranges of a (row, kv head) are neighbours in it, so whatever a workgroup waits
// for is resident or next in line; the polls are bounded all the same.
// ---------------------------------------------------------------------------------
template <int NT, bool POLL>
__device__ __forceinline__ void merge_ranges(const void* phk, size_t sstride, int nsr, uint32_t tag,
                                             int o_lo, int n_out, float* lds, __hip_bfloat16* out_hk SV_TS_PARAM,
                                             [[maybe_unused]] int ts_wg) {
  static_assert(NT == 256 || NT == 128, "thread layout of the merge");
  constexpr int LNT = NT == 256 ? 8 : 7;
  const int tid = threadIdx.x;
  const int lrg = n_out <= 32 ? 3 : n_out <= 64 ? 2 : n_out <= 128 ? 1 : 0;
  const int RG = 1 << lrg, OPP = NT >> lrg;
  float* s_acc = lds;   // [RG][OPP] weighted sums, then the same for reference exponents and weights
  float* s_m = s_acc + NT;
  float* s_w = s_m + NT;
  const int ol = tid & (OPP - 1), rg = tid >> (LNT - lrg);
  for (int ob = 0; ob < n_out; ob += OPP) {
    const int o = o_lo + ob + (ob + ol < n_out ? ol : 0);
    const int g = o >> 7, d = o & (D - 1);
    const unsigned long long* pv = (const unsigned long long*)phk + (size_t)g * PW;   // POLL
    const float* pf = (const float*)phk + (size_t)g * PW;                             // !POLL
    float m_ref = -INFINITY, wsum = 0.f, acc = 0.f;
    [[maybe_unused]] unsigned long long ts_tries = 0;
    // One pass: U ranges per thread, s0, s0 + RG, ...; all but the last are known to exist, the last may lie past
    // the end for the higher range groups (it then reads the thread's first range again and is left out).  The
    // loads are unconditional, so that the compiler issues them together; guarded ones it waits for one by one.
    auto pass = [&](auto Uc, int s0) {
      constexpr int U = decltype(Uc)::value;
      const bool last_ok = s0 + RG * (U - 1) < nsr;
      unsigned long long wv[U], we[U];
      bool ok = false;
      for (int it = 0; it < kPollLimit && !ok; ++it) {
        SV_TS_COUNT(ts_tries);
        if (it >= 3) __builtin_amdgcn_s_sleep(2);
        ok = true;
#pragma unroll
        for (int j = 0; j < U; ++j) {
          const int si = (j < U - 1 || last_ok) ? s0 + RG * j : s0;
          if constexpr (POLL) {
            wv[j] = __hip_atomic_load(pv + (size_t)si * sstride + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            we[j] = __hip_atomic_load(pv + (size_t)si * sstride + D, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          } else {
            wv[j] = __float_as_uint(pf[(size_t)si * sstride + d]);
            we[j] = __float_as_uint(pf[(size_t)si * sstride + D]);
          }
        }
        if constexpr (POLL) {
#pragma unroll
          for (int j = 0; j < U; ++j) ok = ok && (uint32_t)(wv[j] >> 32) == tag && (uint32_t)(we[j] >> 32) == tag;
        }
      }
      float mx = m_ref;
#pragma unroll
      for (int j = 0; j < U; ++j)
        if (j < U - 1 || last_ok) mx = fmaxf(mx, __uint_as_float((uint32_t)we[j]));
      // a read that never saw its tag (the limit is thousands of times any launch's length) poisons the output
      if (!ok) mx = __uint_as_float(0x7fc00000u);
      const float resc = m_ref == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_ref - mx);
      acc *= resc, wsum *= resc;
#pragma unroll
      for (int j = 0; j < U; ++j)
        if (j < U - 1 || last_ok) {
          const float w = __builtin_amdgcn_exp2f(__uint_as_float((uint32_t)we[j]) - mx);
          acc += w * __uint_as_float((uint32_t)wv[j]);
          wsum += w;
        }
      m_ref = mx;
    };
    // ranges per thread: ceil(nsr / RG) for the lowest range groups, one less for the others; whole passes of 8,
    // then ONE pass of exactly what is left
    int left = (nsr + RG - 1) >> lrg, s0 = rg;
    for (; left > 8; left -= 8, s0 += 8 * RG) pass(std::integral_constant<int, 8>{}, s0);
    if (s0 < nsr) {   // (a thread of a higher range group may have nothing at all in the last pass)
      switch (left) {
        case 1: pass(std::integral_constant<int, 1>{}, s0); break;
        case 2: pass(std::integral_constant<int, 2>{}, s0); break;
        case 3: pass(std::integral_constant<int, 3>{}, s0); break;
        case 4: pass(std::integral_constant<int, 4>{}, s0); break;
        case 5: pass(std::integral_constant<int, 5>{}, s0); break;
        case 6: pass(std::integral_constant<int, 6>{}, s0); break;
        case 7: pass(std::integral_constant<int, 7>{}, s0); break;
        default: pass(std::integral_constant<int, 8>{}, s0); break;
      }
    }
    SV_TS(0, ts_wg, 4);
    SV_TS_VAL(ts_wg, 6, ts_tries);
    s_acc[tid] = acc, s_m[tid] = m_ref, s_w[tid] = wsum;   // tid = rg * OPP + ol
    __syncthreads();
    if (2 * tid < OPP && ob + 2 * tid < n_out) {   // two neighbouring dims per thread: one 4-byte store
      const int oo = 2 * tid;
      float mx = -INFINITY;
      for (int k = 0; k < RG; ++k) mx = fmaxf(mx, s_m[k * OPP + oo]);   // a poisoned reference shows in w below
      float t0 = 0.f, t1 = 0.f, wt = 0.f;
      for (int k = 0; k < RG; ++k) {
        const float mk = s_m[k * OPP + oo];
        const float w = mk == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mk - mx);
        t0 += w * s_acc[k * OPP + oo], t1 += w * s_acc[k * OPP + oo + 1];
        wt += w * s_w[k * OPP + oo];
      }
      const float inv = 1.0f / wt;
      const uint32_t w01 = bf_round_bits(t0 * inv) | (bf_round_bits(t1 * inv) << 16);
      *(uint32_t*)(out_hk + o_lo + ob + oo) = w01;   // outputs of a kv head are contiguous: [head in group][128]
    }
    __syncthreads();
  }
}

// The outputs of a (row, kv head) are shared out in runs of 32 among M workgroups; workgroup j of M takes
// [o_lo, o_lo + n_out).  False if it gets none.
__device__ __forceinline__ bool merge_share(int G, int M, int j, int& o_lo, int& n_out) {
  const int n_units = G * 4, upw = (n_units + M - 1) / M;
  o_lo = 32 * min(n_units, j * upw);
  n_out = 32 * min(n_units, j * upw + upw) - o_lo;
  return j < M && n_out > 0;
}

// ONE: a single row (one stream).  Its cache pointers, length and everything else needed to issue the first
// loads are the leading 16 dwords of the argument list, which reach the wavefront in SGPRs at launch (kernel
// argument preload) instead of through a first dependent fetch (a scalar-memory round trip in front of the first
// global load); to fit, the small integers travel in one word (decode_shape) and the head stride as 32 bits.  The
// by-value table, at the end, is not read.
__host__ __device__ inline uint32_t decode_shape(int fused, int rotate, int G, int n_kv_heads, int n_q_heads) {
  return (uint32_t)(fused != 0) | (uint32_t)(rotate != 0) << 1 | (uint32_t)G << 2 | (uint32_t)n_kv_heads << 8 |
         (uint32_t)n_q_heads << 16;   // G <= 8, n_kv_heads <= 255, n_q_heads <= 65535 (checked by the launcher)
}
template <int NW, bool ONE, bool STREAM>
__global__ __launch_bounds__(NW * 64, 2) void k_decode_mfma(__hip_bfloat16* k0_, __hip_bfloat16* v0_, const float2* cs0_,
                                                         int len0_, int keys_per_split,
                                                         const __hip_bfloat16* __restrict__ q,
                                                         const __hip_bfloat16* __restrict__ k_new,
                                                         uint32_t head_stride_elems, uint32_t shape, void* part,
                                                         const __hip_bfloat16* __restrict__ v_new,
                                                         __hip_bfloat16* __restrict__ out, DecTable tab SV_TS_PARAM) {
  const int fused = shape & 1, rotate = (shape >> 1) & 1, G = (shape >> 2) & 15, n_kv_heads = (shape >> 8) & 255,
            n_q_heads = (int)(shape >> 16);
  const int hdr_words = hdr_words_of(n_kv_heads);
  constexpr float c_log2 = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)
  [[maybe_unused]] const int ts_wg = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
  SV_TS(0, ts_wg, 0);
  __shared__ float sO[NW][GMAX][D];                                 // wavefront results (merge)
  __shared__ float sML[NW][GMAX][2];

  const int sp = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  DecRow rd;
  if constexpr (ONE) rd = DecRow{k0_, v0_, cs0_, len0_, keys_per_split, 0};
  else rd = tab.r[b];
  const int len = rd.len;
  const int kps = rd.kps;   // rows of a batch are cut into ranges of their own size
  const int nsr = (len + kps - 1) / kps;   // key ranges of this row
  // Single stream: the words' header of this kv head, {tag of the launch before, its number of key ranges}, written
  // by the launch before (read here, used after the tiles).  This launch's tag is the next one, never 0.
  // The workgroup uses the value thread 0 read, handed round through LDS behind the barrier that precedes all its
  // publishing: the workgroup of range 0 replaces the header once it has seen every range publish, i.e. after every
  // workgroup's thread 0 has read it (a later wavefront of a workgroup might see the new one).
  __shared__ unsigned long long sHdr;
  // (Every thread asks for it, without a branch: behind `if (tid == 0)` the compiler waits for it on the spot.)
  [[maybe_unused]] unsigned long long hdr_old = 0;
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
  // being decoded comes from the caller's buffer.  Rows past the range's end are loaded like the others (planes hold
  // whole 64-key tiles, their scores are replaced by the mask below): no load of a tile sits behind a branch, so the
  // compiler can count the loads issued after the queries' and wait for those alone.
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
        if constexpr (STREAM) kreg[gi][kk] = stream_load(src + 32 * kk);
        else kreg[gi][kk] = *(const uint4*)(src + 32 * kk);
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
  // Memory first, everything below overlaps its latency, and in this order: the query heads and the cos/sin of the
  // rotation, THEN the tile.  Loads return in the order they were issued, so the wavefront can wait for the small ones
  // alone and rotate the queries while K and V are still on their way; issued after the tile they could only be had
  // by waiting for the tile as well, with the rotation's vector work behind the data instead of under it.
  // Query heads of this kv head as the B operand: lane holds head l16, dims 8 lg + 32 kk + j.  Lanes past the group
  // repeat its last head (their columns of the products are never looked at), so the four loads are unconditional and
  // go out together.  (Guarded by l16 < G, the compiler branched around each and waited for the first, and with it
  // for every load before it, to move a register: a memory round trip before the other three were even issued.)
  uint4 qraw[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    qraw[kk] = *(const uint4*)(q + ((size_t)b * n_q_heads + hk * G + min(l16, G - 1)) * D + 8 * lg + 32 * kk);
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
  __builtin_amdgcn_sched_barrier(0);
  {   // (a wavefront without a tile, at the end of a short last range, loads the range's last one and leaves it unused)
    const int t0 = min(wave, max(n_tiles - 1, 0));
    issue_k(k0 + t0 * TK);
    issue_v(k0 + t0 * TK);
  }
  // the wavefront whose tile holds the token being decoded fetches that token's V (one element per head dim for
  // the lanes that will own it) along with its first loads
  // (one element per 32-bit register: packed two to a register, the compiler waits for the loads inside the branch, and
  // with them for every load issued before, to do the packing)
  uint32_t vnew_bits[8] = {};
  const bool owns_new = fused && len - 1 >= k0 && len - 1 < k1 && ((len - 1 - k0) / TK) % NW == wave;
  if (owns_new) {
#pragma unroll
    for (int blk = 0; blk < 8; ++blk) vnew_bits[blk] = *(const unsigned short*)(v_new + new_off + 16 * blk + l16);
  }
  // (the header: asked for here, behind the tile's loads, because `part` is not among the preloaded arguments and
  // fetching it first would put a scalar-memory round trip in front of them)
  if constexpr (ONE) hdr_old = ((const unsigned long long*)part)[hk];
  __builtin_amdgcn_sched_barrier(0);
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
  // One tile.  MORE: the wavefront has a further tile, whose loads go out from inside this one.  The loop below runs
  // the tiles with a successor and then the last one by itself, so that in each of the two bodies the loads in flight
  // are the same on every path and the compiler can wait for K alone while V^T is still on its way (with the
  // prefetch behind a condition it waited for everything).
  auto tile = [&](auto MORE, int t) {
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
          vdst[blk * 16 * kVB] = (unsigned short)vnew_bits[blk];
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
    if constexpr (decltype(MORE)::value) issue_k(kt + NW * TK);
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
    if constexpr (decltype(MORE)::value) issue_v(kt + NW * TK);
  };
  {
    int t = wave;
    for (; t + NW < n_tiles; t += NW) tile(std::true_type{}, t);
    if (t < n_tiles) tile(std::false_type{}, t);
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
  if constexpr (ONE) {
    if (tid == 0) sHdr = hdr_old;
  }
  __syncthreads();
  if constexpr (ONE) hdr_old = sHdr;

  // ---- merge the wavefronts; with one key range this is the result, else the range's partial result: normalised
  // values and the log-sum-exp (log2 units)
  // (a single stream: 64-bit words {value, launch tag} behind the headers, read in this launch; a batch: plain floats
  // for the merge launch)
  const size_t prow_off = ((size_t)(rd.pair0 + sp) * n_q_heads + (size_t)hk * G) * PW;
  unsigned long long* const words = (unsigned long long*)part + hdr_words;
  unsigned long long* prow = words + prow_off;
  float* prow_f = (float*)part + prow_off;
  const uint32_t tag_old = __builtin_amdgcn_readfirstlane((uint32_t)(hdr_old >> 32));   // uniform, and known to be
  const uint32_t tag = tag_old + 1u == 0u ? 1u : tag_old + 1u;
  const unsigned long long tag_hi = (unsigned long long)tag << 32;
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
    const float val = acc / lsum;   // every range holds at least one key: lsum > 0
    if (nsr == 1) {
      out[((size_t)b * n_q_heads + hk * G + g) * D + d] = __float2bfloat16(val);
    } else if constexpr (ONE) {
      __hip_atomic_store(prow + (size_t)g * PW + d, tag_hi | __float_as_uint(val), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
      if (d == 0)
        __hip_atomic_store(prow + (size_t)g * PW + D, tag_hi | __float_as_uint(mn + __log2f(lsum)), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    } else {
      prow_f[(size_t)g * PW + d] = val;
      if (d == 0) prow_f[(size_t)g * PW + D] = mn + __log2f(lsum);
    }
  }
  if constexpr (ONE) {
    // A single stream is latency bound and its workgroups end together: they merge the key ranges themselves, the
    // workgroups of the first min(ranges, 4 G) ranges of a kv head taking a run of outputs each, instead of leaving
    // it to a second launch (a launch gap and a round trip of its own: about 1.2 us more per layer-step).
    // Words of ranges that the launch before had and this one has not (the cache shrank) go back to zero, so that no
    // word is ever older than one launch: a word that does not carry this launch's tag carries the one before or none,
    // also when the 32-bit tag wraps, and nothing depends on host state (a captured launch can be replayed).
    const int nsr_old = (int)(uint32_t)hdr_old;
    for (int r = nsr + sp; r < nsr_old; r += nsr) {
      unsigned long long* pz = words + ((size_t)r * n_q_heads + (size_t)hk * G) * PW;
      for (int idx = tid; idx < G * PW; idx += NW * 64)
        __hip_atomic_store(pz + idx, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (nsr == 1) {
      if (tid == 0) ((unsigned long long*)part)[hk] = tag_hi | 1ull;
      return;
    }
    int o_lo, n_out;
    if (!merge_share(G, min(nsr, G * 4), sp, o_lo, n_out)) return;
    // the first merge read also wants this workgroup's own words: let their stores be acknowledged first (a read
    // that overtakes them costs a second round trip)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    SV_TS(0, ts_wg, 3);
    __syncthreads();   // the wavefront results in LDS have been read: their space is reused
    merge_ranges<NW * 64, true>(words + ((size_t)rd.pair0 * n_q_heads + (size_t)hk * G) * PW, (size_t)n_q_heads * PW, nsr,
                                tag, o_lo, n_out, &sO[0][0][0], out + ((size_t)b * n_q_heads + hk * G) * D SV_TS_ARG(ts_slot),
                                ts_wg);
    // the workgroup of range 0 has seen every range of the kv head publish, i.e. read the header: the new one goes in
    if (sp == 0 && tid == 0) ((unsigned long long*)part)[hk] = tag_hi | (uint32_t)nsr;
#ifdef SV_TIMELINE
    __builtin_amdgcn_s_waitcnt(0x0F70);
    SV_TS(0, ts_wg, 5);
#endif
  }
}

// ---------------------------------------------------------------------------------
// Merge of the key ranges of a batch's rows, as a launch of its own: the rows of a batch end at very different times
// (the first workgroups of a ragged 16-stream batch after 6 us, the last after 36 us), and merging inside the decode
// launch ends later there than this does (measured: the partial results of the last workgroups need about 2.3 us to
// get through a loaded memory system and 1.5 us to come back).  kMergeWGs workgroups per (row, kv head) (14 and
// 28 measured slower on the ragged batch).
// grid: (kMergeWGs, n_kv_heads, n_rows), block: 256 threads.
// ---------------------------------------------------------------------------------
constexpr int kMergeWGs = 7;
struct RangeTable {
  uint32_t row[kMaxRowsD];   // per row: first (row, key range) pair | key ranges << 16.  One 32-bit word, so that the
                             // lookup by a (uniform) row index is ONE scalar load from the kernel arguments; as bytes and
                             // halfwords the compiler fetched the two fields with two dependent vector loads, two memory
                             // round trips in front of the kernel's real loads
};
__global__ __launch_bounds__(256) void k_decode_merge(const float* __restrict__ part,
                                                      __hip_bfloat16* __restrict__ out, int n_q_heads, int G,
                                                      RangeTable rt) {
  __shared__ float lds[3 * 256];
  const int hk = blockIdx.y, b = blockIdx.z;
  const uint32_t row = rt.row[b];
  const int nsr = (int)(row >> 16), pair0 = (int)(row & 0xffffu);
  int o_lo, n_out;
  if (nsr == 1 || !merge_share(G, kMergeWGs, blockIdx.x, o_lo, n_out)) return;   // one range: the decode kernel wrote the output
#ifdef SV_TIMELINE
  constexpr int ts_slot = 0;
#endif
  merge_ranges<256, false>(part + ((size_t)pair0 * n_q_heads + (size_t)hk * G) * PW, (size_t)n_q_heads * PW, nsr, 0u,
                           o_lo, n_out, lds, out + ((size_t)b * n_q_heads + hk * G) * D SV_TS_ARG(ts_slot), 1 << 20);
}

#ifdef SV_TIMELINE
int g_ts_launch = 0;   // host: launches so far; the slot of a launch is this modulo 8
#endif

}  // namespace

// Where the key ranges' partial results go.  marked: header words (hdr_words_of), then the 64-bit words of single-stream
// launches, room for marked_pairs (row, key range) pairs; written by nothing else, zero before the first launch.
// plain: floats of batch launches, plain_pairs pairs.
struct DecScratch {
  unsigned long long* marked;
  int64_t marked_pairs;
  float* plain;
  int64_t plain_pairs;
};

template <int NW>
static hipError_t decode_launch(const sv_cache* c, const DecTable& tab, int fused, int nr, int max_len, int64_t total_tiles,
                         const void* q, const void* k_new, const void* v_new, void* o, size_t r0,
                         const DecScratch& scr, hipStream_t s) {
  const int Hq = c->cfg.n_q_heads, Hkv = c->cfg.n_kv_heads;
  // More than 96 MB of K and V in this launch, one long stream or many: non-temporal loads (rows that are the layers
  // of ONE stream keep the plain loads: their 308 MB are read again at the next token and the Infinity Cache still
  // holds most of them).
  const bool stream_loads = total_tiles * (int64_t)(TK * D * 2 * 2) * Hkv >= ((int64_t)96 << 20);
  const bool one = nr == 1 && !stream_loads;   // the single-stream instantiation: merges its key ranges itself
  const int64_t part_pairs = one ? scr.marked_pairs : scr.plain_pairs;
  // Key ranges.  A single stream is latency bound: ranges of 128 keys (one 32-key tile per wavefront) spread its
  // few hundred tiles over the most CUs and cost one memory round trip.  A batch is bandwidth bound: longer ranges
  // keep the partial results and their merge small, and all workgroups should be resident at once (two fit a CU:
  // 512), since one workgroup more than that and a second, nearly empty round follows the first (measured on 16
  // ragged rows: 516 workgroups 3.6 TB/s, 440 workgroups 4.2 TB/s).  So: the smallest target T, a multiple of 128
  // keys (whole tiles for each of the 4 wavefronts: ranges of 800 keys, 7 tiles for one wavefront and 6 for the
  // others, measured 6 % slower than ranges of 896), for which sum_b ceil(len_b / T) * kv heads <= 512; then every
  // row is cut into ceil(len_b / T) ranges of EQUAL size (rounded up to 128 keys), so that a row does not end in a
  // range much shorter than the others.  (The grid is rows x kv heads x the widest row's ranges, with empty
  // workgroups where a row is shorter; ids go to the 8 XCDs in turn, so depending on the grid's width one XCD can run
  // out of its 64 slots before the launch has 512 workgroups.  A one-dimensional grid over the ranges that exist
  // removes that, 8 rows at 256 workgroups: 35.6 -> 27.5 us, but finding a workgroup's row costs a second dependent
  // read of the arguments, +1.3 us on every launch, and nothing at the 16-row shapes measured here.  Moving rows to
  // the next shorter range length until the slots are full, 508 workgroups on the ragged batch, measured 54 us
  // instead of 40 on this grid (the drop sets in before the 512th workgroup) and level with 440 workgroups on the
  // one-dimensional grid: the choice errs on the side of longer ranges.  More, shorter workgroups than slots, left
  // to the dispatcher (3 or 4 tiles per wavefront, 750 to 1000 workgroups): 43.7 us against 39.3.)
  constexpr int kSlots = 512;
  const int forced = std::min(c->opt[SV_OPT_DECODE_TILES_PER_WAVE], 64);
  if (part_pairs < nr) return hipErrorInvalidValue;   // every row needs at least one pair (callers check their limits)
  int T = forced > 0 ? TK * NW * forced : TK * NW;
  for (;; T += TK * NW) {
    int64_t pairs = 0;
    int widest = 0;
    for (int b = 0; b < nr; ++b) {
      const int nb = (tab.r[b].len + T - 1) / T;
      pairs += nb;
      widest = std::max(widest, nb);
    }
    const bool fits = widest <= kMaxSplitsD && pairs <= part_pairs;   // scratch: one slot per (row, key range)
    if (fits && (forced > 0 || pairs * Hkv <= kSlots || T >= max_len)) break;
  }
  DecTable tabk = tab;
  RangeTable rt = {};
  int n_splits = 1, pair0 = 0;
  for (int b = 0; b < nr; ++b) {
    const int len = tab.r[b].len, nb = std::max(1, (len + T - 1) / T);
    const int kps = ((len + nb - 1) / nb + TK * NW - 1) / (TK * NW) * (TK * NW);
    const int ranges = (len + kps - 1) / kps;   // <= nb <= kMaxSplitsD
    tabk.r[b].kps = kps;
    tabk.r[b].pair0 = pair0;
    rt.row[b] = (uint32_t)pair0 | (uint32_t)ranges << 16;   // pair0 < 2^16: at most kMaxRowsD x kMaxSplitsD pairs
    pair0 += ranges;
    n_splits = std::max(n_splits, ranges);
  }
  void* part = one ? (void*)scr.marked : (void*)scr.plain;
  const int keys_per_split = tabk.r[0].kps;
  if (Hkv > 255 || Hq > 65535 || c->group > GMAX || c->head_stride / 2 > 0xffffffffull) return hipErrorInvalidValue;
  const uint32_t shape = decode_shape(fused, c->cfg.rope_mode != SV_ROPE_NONE, c->group, Hkv, Hq);
  const __hip_bfloat16* qp = (const __hip_bfloat16*)q + r0 * Hq * D;
  const __hip_bfloat16* knp = k_new ? (const __hip_bfloat16*)k_new + r0 * Hkv * D : nullptr;
  const __hip_bfloat16* vnp = v_new ? (const __hip_bfloat16*)v_new + r0 * Hkv * D : nullptr;
  __hip_bfloat16* op = (__hip_bfloat16*)o + r0 * Hq * D;
  const DecRow& r = tabk.r[0];
  if (one)
    hipLaunchKernelGGL((k_decode_mfma<NW, true, false>), dim3(n_splits, Hkv, 1), dim3(NW * 64), 0, s, r.k, r.v, r.cs, r.len,
                       keys_per_split, qp, knp, (uint32_t)(c->head_stride / 2), shape, part, vnp, op, tabk SV_TS_ARG(g_ts_launch % 8));
  else if (stream_loads)
    hipLaunchKernelGGL((k_decode_mfma<NW, false, true>), dim3(n_splits, Hkv, nr), dim3(NW * 64), 0, s, r.k, r.v, r.cs, r.len,
                       keys_per_split, qp, knp, (uint32_t)(c->head_stride / 2), shape, part, vnp, op, tabk SV_TS_ARG(g_ts_launch % 8));
  else
    hipLaunchKernelGGL((k_decode_mfma<NW, false, false>), dim3(n_splits, Hkv, nr), dim3(NW * 64), 0, s, r.k, r.v, r.cs, r.len,
                       keys_per_split, qp, knp, (uint32_t)(c->head_stride / 2), shape, part, vnp, op, tabk SV_TS_ARG(g_ts_launch % 8));
#ifdef SV_TIMELINE
  ++g_ts_launch;
#endif
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_splits == 1 || one) return e;
  hipLaunchKernelGGL(k_decode_merge, dim3(kMergeWGs, Hkv, nr), dim3(256), 0, s, scr.plain, op, Hq, c->group, rt);
  return hipGetLastError();
}

// Partial results of the key ranges live in the cache arena by default; sv_attn_decode_static keeps them in a
// file-scope device array instead (callers that cannot provide scratch memory; zero at load, as every device-scope
// array): its first half holds the marked words of single-stream launches, its second half the floats of batches.
// The array's name is only a host-side handle: its device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kMaxDevices] = {};

static hipError_t static_scratch_of_device(void** ptr_out, int* dev_out) {
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
  if (dev_out) *dev_out = dev;
  return hipSuccess;
}

hipError_t decode_static_scratch(void** ptr_out) { return static_scratch_of_device(ptr_out, nullptr); }

size_t decode_marked_bytes(const sv_config& cfg) {
  return ((size_t)kMaxSplitsD * cfg.n_q_heads * PW + hdr_words_of(cfg.n_kv_heads)) * sizeof(unsigned long long);
}

int64_t decode_plain_pairs(const sv_cache* c) {   // the arena's split-KV region holds part_rows x heads x 128 floats
  return c->part_rows * D / PW;
}

int64_t decode_static_pairs(const sv_cache* c) {
  return (int64_t)(kStaticScratchBytes / 2 / ((size_t)c->cfg.n_q_heads * PW * sizeof(float)));
}

// len_one / cs_one (single row only, 0 / NULL = the stream's own): the row's visible length and the cos/sin of its
// query token, for a token of a run that was registered as a whole and is decoded one token at a time.
static hipError_t decode_rows(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused, const void* q,
                              const void* k_new, const void* v_new, void* o, const DecScratch& scr, hipStream_t s,
                              int64_t len_one = 0, const float2* cs_one = nullptr) {
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
      const int64_t len = n_list == 1 && len_one > 0 ? len_one : st.len;
      tab.r[b].len = (int)len;
      tab.r[b].cs = n_list == 1 && cs_one ? cs_one : c->last_cs + (size_t)sid * (D / 2);
      max_len = std::max(max_len, (int)len);
      if (layer >= 0) total_tiles += (len + TK - 1) / TK;
    }
    hipError_t e = decode_launch<4>(c, tab, fused, nr, max_len, total_tiles, q, k_new, v_new, o, (size_t)r0, scr, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_attn_decode_mfma(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused,
                                   const void* q, const void* k_new, const void* v_new, void* o, hipStream_t s) {
  const DecScratch scr = {c->part_dec, kMaxSplitsD, c->part_o, decode_plain_pairs(c)};
  return decode_rows(c, layer, streams, n_list, fused, q, k_new, v_new, o, scr, s);
}

hipError_t launch_decode_step_of_run(const sv_cache* c, int layer, int stream, int64_t len, int run_index, const void* q,
                                     const void* k_new, const void* v_new, void* o, hipStream_t s) {
  const DecScratch scr = {c->part_dec, kMaxSplitsD, c->part_o, decode_plain_pairs(c)};
  const int32_t sid = stream;
  const float2* cs = c->cs_tab + ((size_t)stream * c->cfg.max_q_tokens + run_index) * (D / 2);
  return decode_rows(c, layer, &sid, 1, 1, q, k_new, v_new, o, scr, s, len, cs);
}

hipError_t launch_attn_decode_mfma_static(const sv_cache* c, int layer, const int32_t* streams, int n_list,
                                          const void* q, void* o, hipStream_t s) {
  void* p = nullptr;
  int dev = 0;
  hipError_t e = static_scratch_of_device(&p, &dev);
  if (e != hipSuccess) return e;
  const size_t half = kStaticScratchBytes / 2;
  const DecScratch scr = {(unsigned long long*)p,
                          (int64_t)((half - (size_t)hdr_words_of(c->cfg.n_kv_heads) * 8) / ((size_t)c->cfg.n_q_heads * PW * sizeof(unsigned long long))),
                          (float*)((char*)p + half), decode_static_pairs(c)};
  return decode_rows(c, layer, streams, n_list, 0, q, nullptr, nullptr, o, scr, s);
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
