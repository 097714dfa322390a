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
// Eviction scan, one workgroup of 16 wavefronts per stream.
//
// keep(i)  : text  -> rank < n_sink or rank >= text_lo     (sink + recent text)
//            vision-> rank >= vis_lo                         (recent vision)
// dst(i)   : exclusive prefix count of keep
// base'(i) : exclusive prefix sum over kept tokens of the position advance, where a
//            text token advances by 1 and a vision block advances by its extent at
//            its last retained token.  With every token its own block of extent 1
//            (1-D mode) base' equals dst.
// Survivors' metadata is written compacted to `out`; src[dst] = i is the gather
// list for the K/V move and delta[dst] = base - base' the shift for the re-rotation.
//
// A pass covers kScanSub x 1024 tokens: sub-tile k holds tokens base + 1024 k + tid, so every load is coalesced
// and all loads of a pass are independent and issued together (one memory round trip per 4096 tokens instead of
// one per 1024).  Within a sub-tile a wavefront's keep count comes from the ballot and a popcount, its advances
// from a shuffle scan; the 64 (sub-tile, wavefront) totals of a pass go through LDS and are scanned by the first
// wavefront, and a running carry links the passes.
// ---------------------------------------------------------------------------------
constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kScanSub = 4;

__device__ __forceinline__ bool keep_rule(int type, int64_t rank, int64_t n_sink, int64_t text_lo, int64_t vis_lo) {
  return type == SV_TEXT ? (rank < n_sink || rank >= text_lo) : (rank >= vis_lo);
}

__global__ __launch_bounds__(kScanThreads) void k_evict_scan(MetaPtrs in, MetaPtrs out, int32_t* __restrict__ src,
                                                             int32_t* __restrict__ delta,
                                                             int32_t* __restrict__ next_out,
                                                             int32_t* __restrict__ n_out, int n_old, int64_t n_sink,
                                                             int64_t text_lo, int64_t vis_lo) {
  __shared__ int sh_cnt[kScanSub * kScanWaves];
  __shared__ int sh_adv[kScanSub * kScanWaves];
  __shared__ int sh_tot[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int carry_cnt = 0, carry_adv = 0;
  for (int base = 0; base < n_old; base += kScanThreads * kScanSub) {
    int type[kScanSub], blk[kScanSub], old_base[kScanSub], type_n[kScanSub], blk_n[kScanSub];
    int64_t rank[kScanSub], gid[kScanSub], rank_n[kScanSub];
    short4 loc[kScanSub];
#pragma unroll
    for (int k = 0; k < kScanSub; ++k) {   // the token and its successor (the look-ahead for "last of its block")
      const unsigned i = (unsigned)(base + k * kScanThreads + tid);   // (unsigned: scalar base + 32-bit lane offset)
      const bool valid = i < (unsigned)n_old, valid_n = i + 1 < (unsigned)n_old;
      type[k] = valid ? in.type[i] : SV_TEXT;
      rank[k] = valid ? in.rank[i] : 0;
      blk[k] = valid ? in.blk[i] : -1;
      gid[k] = valid ? in.gid[i] : 0;
      loc[k] = valid ? in.local4[i] : make_short4(0, 0, 0, 1);
      old_base[k] = valid ? in.pos4[i].w : 0;
      type_n[k] = valid_n ? in.type[i + 1] : SV_TEXT;
      rank_n[k] = valid_n ? in.rank[i + 1] : 0;
      blk_n[k] = valid_n ? in.blk[i + 1] : -2;   // matches no block
    }
    bool keep[kScanSub];
    int adv[kScanSub], lane_cnt[kScanSub], incl[kScanSub];
#pragma unroll
    for (int k = 0; k < kScanSub; ++k) {
      const int i = base + k * kScanThreads + tid;
      keep[k] = i < n_old && keep_rule(type[k], rank[k], n_sink, text_lo, vis_lo);
      adv[k] = 0;
      if (keep[k]) {
        if (type[k] == SV_TEXT) {
          adv[k] = 1;
        } else {
          // last retained token of its vision block?  (a token without a block, blk < 0, is its own block)
          const bool next_stays = blk[k] >= 0 && blk_n[k] == blk[k] && i + 1 < n_old &&
                                  keep_rule(type_n[k], rank_n[k], n_sink, text_lo, vis_lo);
          adv[k] = next_stays ? 0 : (int)loc[k].w;
        }
      }
      // wavefront level: ballot/popcount for the count, shuffle scan for the advance
      const unsigned long long bal = __ballot(keep[k]);
      lane_cnt[k] = __popcll(bal & ((1ull << lane) - 1ull));
      incl[k] = adv[k];
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(incl[k], off);
        if (lane >= off) incl[k] += y;
      }
      if (lane == 63) {
        sh_cnt[k * kScanWaves + wave] = __popcll(bal);
        sh_adv[k * kScanWaves + wave] = incl[k];
      }
    }
    __syncthreads();
    // exclusive prefix over the kScanSub * 16 = 64 (sub-tile, wavefront) segments in token order (segment
    // k * 16 + w), by the first wavefront: one segment per lane
    static_assert(kScanSub * kScanWaves == 64, "one segment per lane of the first wavefront");
    if (wave == 0) {
      const int c0 = sh_cnt[lane], a0 = sh_adv[lane];
      int ci = c0, ai = a0;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int yc = __shfl_up(ci, off), ya = __shfl_up(ai, off);
        if (lane >= off) ci += yc, ai += ya;
      }
      sh_cnt[lane] = carry_cnt + ci - c0;
      sh_adv[lane] = carry_adv + ai - a0;
      if (lane == 63) {
        sh_tot[0] = carry_cnt + ci;
        sh_tot[1] = carry_adv + ai;
      }
    }
    __syncthreads();
    int seg_cnt[kScanSub], seg_adv[kScanSub];
#pragma unroll
    for (int k = 0; k < kScanSub; ++k) {
      seg_cnt[k] = sh_cnt[k * kScanWaves + wave];
      seg_adv[k] = sh_adv[k * kScanWaves + wave];
    }
    const int run_cnt = sh_tot[0], run_adv = sh_tot[1];
#pragma unroll
    for (int k = 0; k < kScanSub; ++k) {
      if (keep[k]) {
        const int d = seg_cnt[k] + lane_cnt[k];
        const int nb = seg_adv[k] + (incl[k] - adv[k]);
        out.gid[d] = gid[k];
        out.rank[d] = rank[k];
        out.type[d] = (uint8_t)type[k];
        out.blk[d] = blk[k];
        out.local4[d] = loc[k];
        out.pos4[d] = make_int4(nb + loc[k].x, nb + loc[k].y, nb + loc[k].z, nb);
        src[d] = base + k * kScanThreads + tid;
        delta[d] = old_base[k] - nb;
      }
    }
    carry_cnt = run_cnt;
    carry_adv = run_adv;
    __syncthreads();
  }
  if (tid == 0) {
    *next_out = carry_adv;
    *n_out = carry_cnt;
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
  hipLaunchKernelGGL(k_evict_scan, dim3(1), dim3(kScanThreads), 0, s, in, out, c->src + off, c->delta + off,
                     c->next_pos + 2 * stream + (next_parity ^ 1), c->n_dev + stream, (int)n_old, n_sink, text_lo,
                     vis_lo);
  return hipGetLastError();
}

}  // namespace sv
