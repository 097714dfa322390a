// Integer side of the path: registering new tokens, and the eviction scan that
// turns the three budgets of Sec. 2.1 into a gather list plus new contiguous
// positions (Sec. 2.1, "Contiguous RoPE").  Everything here is exact integer work.

#include "sv_internal.h"

namespace sv {
namespace {

// ---------------------------------------------------------------------------------
// New tokens: slot, arrival id, rank within type, block coordinates and position.
// The scalar position counter lives in device memory as a two-entry ping-pong
// (read next_in, write next_out) so that no thread can read a value another
// block has already advanced.
// ---------------------------------------------------------------------------------
__global__ void k_meta_append(MetaPtrs m, const int32_t* __restrict__ next_in, int32_t* __restrict__ next_out,
                              int64_t slot0, int n, int64_t gid0, int64_t rank_text0, int64_t rank_vis0,
                              int type_uniform, TypeMask mask, int rope3d, int blk, int gT, int gH, int gW,
                              float2* __restrict__ last_cs, const double* __restrict__ inv_freq, int half,
                              int rope_none, int s0, int s01, int f32_data, int32_t* __restrict__ n_dev,
                              float2* __restrict__ cs_tab) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int next = *next_in;
  if (cs_tab != nullptr && j < n * half) {
    // cos/sin of every new token's rotary angles (thread = one token, one frequency), as the row movers compute
    // them: angle in double, sincosf of its float value (the table serves bf16 caches only)
    const int tok = j / half, i = j % half;
    int p;
    if (rope3d && blk >= 0) {
      const int lt = tok / (gH * gW), lh = (tok / gW) % gH, lw = tok % gW;
      p = next + (i < s0 ? lt : (i < s01 ? lh : lw));
    } else {
      p = rope3d ? next + tok : (int)(slot0 + tok);
    }
    float2 cs;
    sincosf((float)((double)p * inv_freq[i]), &cs.y, &cs.x);
    cs_tab[j] = cs;
  }
  if (blockIdx.x == 0 && threadIdx.x < half) {
    // cos/sin of the rotary angles of the LAST token of this append (the decode kernel's query token)
    const int i = threadIdx.x;
    int pt, ph, pw;
    if (rope3d && blk >= 0) pt = next + gT - 1, ph = next + gH - 1, pw = next + gW - 1;
    else pt = ph = pw = rope3d ? next + n - 1 : (int)(slot0 + n - 1);
    const int p = !rope3d ? pt : (i < s0 ? pt : (i < s01 ? ph : pw));
    const double ang = rope_none ? 0.0 : (double)p * inv_freq[i];
    float2 cs;
    if (f32_data) {
      double sd, cd;
      sincos(ang, &sd, &cd);
      cs = make_float2((float)cd, (float)sd);
    } else {
      sincosf((float)ang, &cs.y, &cs.x);
    }
    last_cs[i] = cs;
  }
  if (j == 0) {
    int adv;
    if (!rope3d) adv = (int)(slot0 + n) - next;  // 1-D: position == slot
    else if (blk >= 0) adv = max(gT, max(gH, gW));
    else adv = n;
    *next_out = next + adv;
    *n_dev = (int32_t)(slot0 + n);   // the device's own token count (cross-checked by sv_cache_retained)
  }
  if (j >= n) return;
  int type;
  int64_t rank;
  if (type_uniform >= 0) {
    type = type_uniform;
    rank = (type == SV_TEXT ? rank_text0 : rank_vis0) + j;
  } else {
    type = (mask.w[j >> 5] >> (j & 31)) & 1;
    int vis_before = 0;
    for (int w = 0; w < (j >> 5); ++w) vis_before += __popc(mask.w[w]);
    vis_before += __popc(mask.w[j >> 5] & ((1u << (j & 31)) - 1u));
    rank = type == SV_VISION ? rank_vis0 + vis_before : rank_text0 + (j - vis_before);
  }
  const int64_t slot = slot0 + j;
  m.gid[slot] = gid0 + j;
  m.rank[slot] = rank;
  m.type[slot] = (uint8_t)type;
  if (rope3d && blk >= 0) {
    const int lt = j / (gH * gW), lh = (j / gW) % gH, lw = j % gW;
    m.blk[slot] = blk;
    m.local4[slot] = make_short4((short)lt, (short)lh, (short)lw, (short)max(gT, max(gH, gW)));
    m.pos4[slot] = make_int4(next + lt, next + lh, next + lw, next);
  } else {
    const int p = rope3d ? next + j : (int)slot;
    m.blk[slot] = -1;
    m.local4[slot] = make_short4(0, 0, 0, 1);
    m.pos4[slot] = make_int4(p, p, p, p);
  }
}

// ---------------------------------------------------------------------------------
// Eviction scan, several workgroups per stream.
//
// keep(i)  : text  -> rank < n_sink or rank >= text_lo     (sink + recent text)
//            vision-> rank >= vis_lo                         (recent vision)
// dst(i)   : exclusive prefix count of keep
// base'(i) : exclusive prefix sum over kept tokens of the position advance, where a
//            text token advances by 1 and a vision block advances by its extent at
//            its last retained token.  With every token its own block of extent 1
//            (1-D mode) base' equals dst.
// Survivors' metadata is written compacted to `out`; src[dst] = i is the gather
// list for the K/V move, delta[dst] = base - base' the shift for the re-rotation, and
// dtab[dst][pair] = (cos, -sin) of delta * inv_freq[pair] (rows with delta != 0 only:
// the mover reads no others), i.e. moving from old to new position turns pair i by
// -(delta * inv_freq[i]); stored so that the mover applies the formula of a forward
// rotation.  delta is one scalar per token even in 3-D mode because t, h and w shift together.
//
// Workgroup w owns the tokens [w * span, (w + 1) * span), span = passes x 256, one token per thread and pass.
//   1. It counts its kept tokens and their advances (within a wavefront: ballot + popcount, shuffle sum) and
//      publishes the two totals as 64-bit words {value, launch tag} with relaxed device-scope atomic stores.
//   2. Its first wavefront reads the words of all workgroups before it, again and again until each carries this
//      launch's tag (a word is its own ready flag: a 64-bit access is single-copy atomic and a word is written once
//      per launch; the writers wait for nothing and are dispatched earlier), and sums them: the carry.
//      The tag lives in device memory behind the words: a launch uses the stored value + 1 (never 0), and the last
//      workgroup, which ends only after every other one has published, i.e. read the tag, stores the new value and
//      zeroes the words of the workgroups this launch did not have; so a word left over from an earlier launch
//      carries the tag before this one or none, and nothing depends on host state (a captured launch can be replayed).
//   3. It scans its own tokens (ballot / popcount for the slot, shuffle scan for the advance, four wavefront totals
//      through LDS) on top of the carry and writes the survivors' metadata.
//   4. The kept tokens of a wavefront sit in consecutive slots; their shifts are nearly always one value, so a
//      wavefront evaluates the 64 sincos of a shift once (lane = rotary pair, angle in double) whenever the shift
//      changes along its tokens and writes a 512-byte table row per token.
// At most kScanMaxWG workgroups: longer caches take several passes per workgroup.
// ---------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kScanPollLimit = 1 << 16;

struct ScanTok {
  int type, blk, old_base, type_n, blk_n;
  int64_t rank, gid, rank_n;
  short4 loc;
};

__global__ __launch_bounds__(kScanThreads) void k_evict_scan(MetaPtrs in, MetaPtrs out, int32_t* __restrict__ src,
                                                             int32_t* __restrict__ delta, float2* __restrict__ dtab,
                                                             const double* __restrict__ inv_freq, int half,
                                                             int f32_data, int32_t* __restrict__ next_out,
                                                             int32_t* __restrict__ n_out, int n_old, int64_t n_sink,
                                                             int64_t text_lo, int64_t vis_lo, int passes,
                                                             unsigned long long* agg) {
  __shared__ int sh_cnt[kScanWaves];
  __shared__ int sh_adv[kScanWaves];
  __shared__ int sh_carry[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int w = blockIdx.x, span = passes * kScanThreads;
  const int first = w * span;
  const uint32_t tag_old = (uint32_t)agg[2 * kScanMaxWG];   // written by the launch before this one
  const uint32_t tag = tag_old + 1u == 0u ? 1u : tag_old + 1u;

  // The token and its successor (the look-ahead for "last of its block").  Indices are clamped instead of guarded
  // and the rule below is written without short-circuits, so that every load is unconditional and all nine go out
  // together: guarded, the compiler sinks each load into the branch that uses it, one memory round trip after another.
  auto load_tok = [&](int i) {
    ScanTok t;
    const int ic = min(i, n_old - 1), in_ = min(i + 1, n_old - 1);
    t.type = in.type[ic];
    t.rank = in.rank[ic];
    t.blk = in.blk[ic];
    t.gid = in.gid[ic];
    t.loc = in.local4[ic];
    t.old_base = in.pos4[ic].w;
    t.type_n = in.type[in_];
    t.rank_n = in.rank[in_];
    t.blk_n = in.blk[in_];
    return t;
  };
  auto kept = [&](int type, int64_t rank) {
    const bool text_ok = (rank < n_sink) | (rank >= text_lo), vis_ok = rank >= vis_lo;
    return type == SV_TEXT ? text_ok : vis_ok;
  };
  auto eval = [&](const ScanTok& t, int i, bool& keep, int& adv) {
    keep = (i < n_old) & kept(t.type, t.rank);
    // last retained token of its vision block?  (a token without a block, blk < 0, is its own block)
    const bool next_stays = (t.blk >= 0) & (t.blk_n == t.blk) & (i + 1 < n_old) & kept(t.type_n, t.rank_n);
    const int adv_vis = next_stays ? 0 : (int)t.loc.w;
    adv = keep ? (t.type == SV_TEXT ? 1 : adv_vis) : 0;
  };
  auto wave_sum = [&](int x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    return x;
  };

  // ---- 1. totals of this workgroup's tokens
  const ScanTok t0 = load_tok(first + tid);   // pass 0 stays in registers for step 3
  int my_cnt = 0, my_adv = 0;
  for (int p = 0; p < passes; ++p) {
    const int i = first + p * kScanThreads + tid;
    const ScanTok t = p == 0 ? t0 : load_tok(i);
    bool keep;
    int adv;
    eval(t, i, keep, adv);
    my_cnt += keep ? 1 : 0;
    my_adv += adv;
  }
  my_cnt = wave_sum(my_cnt), my_adv = wave_sum(my_adv);
  if (lane == 0) sh_cnt[wave] = my_cnt, sh_adv[wave] = my_adv;
  __syncthreads();
  const unsigned long long tag_hi = (unsigned long long)tag << 32;
  if (tid == 0) {
    int tc = 0, ta = 0;
#pragma unroll
    for (int k = 0; k < kScanWaves; ++k) tc += sh_cnt[k], ta += sh_adv[k];
    __hip_atomic_store(agg + 2 * w, tag_hi | (uint32_t)tc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(agg + 2 * w + 1, tag_hi | (uint32_t)ta, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // ---- 2. carry: totals of all workgroups before this one
  if (wave == 0) {
    int cc = 0, ca = 0;
    bool lost = false;
    for (int b0 = 0; b0 < w; b0 += 64) {
      const int b = b0 + lane;
      unsigned long long wc = tag_hi, wa = tag_hi;
      for (int it = 0; it < kScanPollLimit; ++it) {
        if (b < w) {
          wc = __hip_atomic_load(agg + 2 * b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          wa = __hip_atomic_load(agg + 2 * b + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if ((uint32_t)(wc >> 32) == tag && (uint32_t)(wa >> 32) == tag) break;
        if (it == kScanPollLimit - 1) lost = true;
        __builtin_amdgcn_s_sleep(1);
      }
      cc += (int)(uint32_t)wc, ca += (int)(uint32_t)wa;
    }
    cc = wave_sum(cc), ca = wave_sum(ca);
    // a word that never showed its tag (the limit is far beyond any launch's length): this workgroup writes
    // nothing, and the failure shows in the device's own token count, which sv_cache_retained checks against the host's
    if (__any(lost)) cc = -1;
    if (lane == 0) sh_carry[0] = cc, sh_carry[1] = ca;
  }
  __syncthreads();
  int run_cnt = sh_carry[0], run_adv = sh_carry[1];
  if (run_cnt < 0) {
    if (tid == 0) *n_out = -1;
    return;
  }

  // ---- 3. and 4. scan of the own tokens on top of the carry, survivors out, table rows
  for (int p = 0; p < passes; ++p) {
    const int i = first + p * kScanThreads + tid;
    const ScanTok t = p == 0 ? t0 : load_tok(i);
    bool keep;
    int adv;
    eval(t, i, keep, adv);
    const unsigned long long bal = __ballot(keep);
    const int lane_cnt = __popcll(bal & ((1ull << lane) - 1ull));
    int incl = adv;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    __syncthreads();   // the totals of the pass before (or of step 1) have been read
    if (lane == 63) sh_cnt[wave] = __popcll(bal), sh_adv[wave] = incl;
    __syncthreads();
    int seg_cnt = run_cnt, seg_adv = run_adv;
#pragma unroll
    for (int k = 0; k < kScanWaves; ++k) {
      if (k < wave) seg_cnt += sh_cnt[k], seg_adv += sh_adv[k];
      run_cnt += sh_cnt[k], run_adv += sh_adv[k];
    }
    const int d = seg_cnt + lane_cnt;
    const int nb = seg_adv + (incl - adv);
    const int dlt = t.old_base - nb;
    if (keep) {
      out.gid[d] = t.gid;
      out.rank[d] = t.rank;
      out.type[d] = (uint8_t)t.type;
      out.blk[d] = t.blk;
      out.local4[d] = t.loc;
      out.pos4[d] = make_int4(nb + t.loc.x, nb + t.loc.y, nb + t.loc.z, nb);
      src[d] = i;
      delta[d] = dlt;
    }
    if (dtab != nullptr) {
      const double my_freq = lane < half ? inv_freq[lane] : 0.0;
      unsigned long long m = __ballot(keep && dlt != 0);
      int cur = 0;
      float2 cs = make_float2(1.f, 0.f);
      while (m) {   // uniform over the wavefront
        const int l = __ffsll((long long)m) - 1;
        m &= m - 1;
        const int dq = __builtin_amdgcn_readlane(dlt, l), dd = __builtin_amdgcn_readlane(d, l);   // l is uniform
        if (dq != cur) {
          cur = dq;
          if (lane < half) {
            const double ang = (double)dq * my_freq;
            if (f32_data) {
              double sd, cd;
              sincos(ang, &sd, &cd);
              cs = make_float2((float)cd, (float)-sd);
            } else {
              // bf16 rows: float accuracy is ample, and the double-precision sincos with its large-argument reduction
              // costs microseconds per call; the angle is reduced to [-pi, pi] in double first (error ~1e-13)
              const double turns = rint(ang * 0.15915494309189535);
              const float r = (float)fma(turns, -6.283185307179586, ang);
              float sf, cf;
              sincosf(r, &sf, &cf);
              cs = make_float2(cf, -sf);
            }
          }
        }
        if (lane < half) dtab[(size_t)dd * half + lane] = cs;
      }
    }
  }
  if (w == (int)gridDim.x - 1) {
    if (tid == 0) {
      *next_out = run_adv;
      *n_out = run_cnt;
      agg[2 * kScanMaxWG] = tag;
    }
    for (int b = (int)gridDim.x + tid; b < kScanMaxWG; b += kScanThreads) agg[2 * b] = 0ull, agg[2 * b + 1] = 0ull;
  }
}

}  // namespace

hipError_t launch_meta_append(const sv_cache* c, int stream, int next_parity, int64_t slot0, int n,
                              int64_t gid0, int64_t rank_text0, int64_t rank_vis0, int type_uniform,
                              const TypeMask* mask, int blk, int gT, int gH, int gW, bool with_cs_tab, hipStream_t s) {
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  MetaPtrs m = c->meta[c->st[stream].cur];
  m.gid += off, m.rank += off, m.pos4 += off, m.local4 += off, m.blk += off, m.type += off;
  TypeMask mk = {};
  if (mask) mk = *mask;
  const int half = c->cfg.head_dim / 2;
  const int threads = 256, blocks = ((with_cs_tab ? n * half : n) + threads - 1) / threads;
  const int32_t* nin = c->next_pos + 2 * stream + next_parity;
  int32_t* nout = c->next_pos + 2 * stream + (next_parity ^ 1);
  hipLaunchKernelGGL(k_meta_append, dim3(blocks), dim3(threads), 0, s, m, nin, nout, slot0, n, gid0, rank_text0,
                     rank_vis0, type_uniform, mk, c->cfg.rope_mode == SV_ROPE_3D ? 1 : 0, blk, gT, gH, gW,
                     c->last_cs + (size_t)stream * half, c->inv_freq, half, c->cfg.rope_mode == SV_ROPE_NONE ? 1 : 0,
                     c->cfg.mrope_sections[0], c->cfg.mrope_sections[0] + c->cfg.mrope_sections[1],
                     c->cfg.dtype == SV_DTYPE_F32 ? 1 : 0, c->n_dev + stream,
                     with_cs_tab ? c->cs_tab + (size_t)stream * c->cfg.max_q_tokens * half : nullptr);
  return hipGetLastError();
}

hipError_t launch_evict_scan(const sv_cache* c, int stream, int next_parity, int64_t n_old, int64_t n_sink,
                             int64_t text_lo, int64_t vis_lo, hipStream_t s) {
  const size_t off = (size_t)stream * (size_t)c->cfg.capacity_tokens;
  const int cur = c->st[stream].cur;
  MetaPtrs in = c->meta[cur], out = c->meta[cur ^ 1];
  in.gid += off, in.rank += off, in.pos4 += off, in.local4 += off, in.blk += off, in.type += off;
  out.gid += off, out.rank += off, out.pos4 += off, out.local4 += off, out.blk += off, out.type += off;
  const int half = c->cfg.head_dim / 2;
  const int tiles = (int)((n_old + kScanThreads - 1) / kScanThreads);
  const int passes = (tiles + kScanMaxWG - 1) / kScanMaxWG;
  const int wgs = (tiles + passes - 1) / passes;
  unsigned long long* agg = c->scan_agg + (size_t)stream * 2 * (kScanMaxWG + 1);
  hipLaunchKernelGGL(k_evict_scan, dim3(wgs), dim3(kScanThreads), 0, s, in, out, c->src + off, c->delta + off,
                     c->cfg.rope_mode != SV_ROPE_NONE ? c->dtab + off * half : nullptr, c->inv_freq, half,
                     c->cfg.dtype == SV_DTYPE_F32 ? 1 : 0, c->next_pos + 2 * stream + (next_parity ^ 1), c->n_dev + stream, (int)n_old, n_sink, text_lo,
                     vis_lo, passes, agg);
  return hipGetLastError();
}

}  // namespace sv
