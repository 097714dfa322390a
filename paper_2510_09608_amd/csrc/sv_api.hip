// Host side of libsv: argument checking, bookkeeping and kernel sequencing.
// All device work is done by the kernels in the sibling translation units; this
// file holds no arithmetic of the method beyond counting which tokens survive.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <new>

#include "sv_internal.h"

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// bf16, head_dim 128, at most 8 query heads per kv head (and at most 255 kv heads: the kernels carry the head
// counts in one packed argument word) and no SV_FLAG_GENERIC_KERNELS: the matrix-core kernels
bool mfma_eligible(const sv_config& c) {
  return c.dtype == SV_DTYPE_BF16 && c.head_dim == 128 && c.n_q_heads / c.n_kv_heads <= 8 && c.n_kv_heads <= 255 &&
         !(c.flags & SV_FLAG_GENERIC_KERNELS);
}

bool config_ok(const sv_config* c) {
  if (!c) return false;
  if (c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_streams < 1) return false;
  if (c->n_q_heads % c->n_kv_heads != 0) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->dtype != SV_DTYPE_F32 && c->dtype != SV_DTYPE_BF16) return false;
  if (c->rope_mode != SV_ROPE_1D && c->rope_mode != SV_ROPE_3D && c->rope_mode != SV_ROPE_NONE) return false;
  // slot and element indices inside the kernels are 32-bit: 2^24 slots x head_dim 128 stays far below 2^31
  if (c->capacity_tokens < 1 || c->capacity_tokens > (int64_t)1 << 24) return false;
  if (c->flags & ~(int32_t)(SV_FLAG_GENERIC_KERNELS | SV_FLAG_HOST_LOGIC_ONLY)) return false;
  if (c->max_q_tokens < 1) return false;
  if (c->rope_mode != SV_ROPE_NONE && !(c->rope_theta > 0.0)) return false;
  if (c->rope_mode == SV_ROPE_3D) {
    int64_t s = 0;
    for (int i = 0; i < 3; ++i) {
      if (c->mrope_sections[i] < 0) return false;
      s += c->mrope_sections[i];
    }
    if (s != c->head_dim / 2) return false;
  }
  return true;
}

// Byte offsets of every region of the arena, in one place so that
// sv_cache_bytes and sv_cache_create cannot disagree.
struct Layout {
  size_t kv, meta_gid[2], meta_rank[2], meta_pos[2], meta_local[2], meta_blk[2], meta_type[2];
  size_t src, delta, dtab, next_pos, n_dev, inv_freq, last_cs, cs_tab, part_o, part_ml, counters, part_dec, scan_agg, total;
  int64_t part_rows;
  size_t part_dec_bytes;
};

Layout make_layout(const sv_config& c) {
  Layout L{};
  const size_t es = c.dtype == SV_DTYPE_F32 ? 4 : 2;
  const size_t cap = (size_t)c.capacity_tokens, S = (size_t)c.n_streams;
  const size_t cap_pad = (cap + 63) / 64 * 64;   // K/V planes hold whole 64-key tiles
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes);
    return o;
  };
  L.kv = take(S * 2 * (size_t)c.n_layers * 2 * (size_t)c.n_kv_heads * cap_pad * (size_t)c.head_dim * es);
  for (int h = 0; h < 2; ++h) {
    L.meta_gid[h] = take(S * cap * 8);
    L.meta_rank[h] = take(S * cap * 8);
    L.meta_pos[h] = take(S * cap * 16);
    L.meta_local[h] = take(S * cap * 8);
    L.meta_blk[h] = take(S * cap * 4);
    L.meta_type[h] = take(S * cap);
  }
  L.src = take(S * cap * 4);
  L.delta = take(S * cap * 4);
  L.dtab = take(S * cap * (size_t)(c.head_dim / 2) * 8);
  L.next_pos = take(S * 2 * 4);
  L.n_dev = take(S * 4);
  L.inv_freq = take((size_t)(c.head_dim / 2) * 8);
  L.last_cs = take(S * (size_t)(c.head_dim / 2) * 8);
  L.cs_tab = take(S * (size_t)c.max_q_tokens * (size_t)(c.head_dim / 2) * 8);
  L.part_rows = std::max<int64_t>(64 * (int64_t)c.n_streams, std::max<int64_t>(4096, 4 * (int64_t)c.max_q_tokens));
  L.part_o = take((size_t)L.part_rows * c.n_q_heads * c.head_dim * 4);
  L.part_ml = take((size_t)L.part_rows * c.n_q_heads * 4 * 4);   // up to 4 floats per (row, range, head)
  L.counters = take((size_t)L.part_rows * c.n_kv_heads * 4);
  // matrix-core decode, single stream: marked words of up to 128 key ranges
  L.part_dec_bytes = mfma_eligible(c) ? sv::decode_marked_bytes(c) : 0;
  L.part_dec = take(L.part_dec_bytes);
  L.scan_agg = take(S * 2 * (sv::kScanMaxWG + 1) * 8);
  L.total = off;
  return L;
}

bool stream_ok(const sv_cache* c, int s) { return c && s >= 0 && s < c->cfg.n_streams; }
bool st_cs_valid(const sv_cache* c, int s) { return c->st[s].cs_tab_valid; }

int64_t iv_count(const std::vector<std::pair<int64_t, int64_t>>& iv) {
  int64_t n = 0;
  for (auto& p : iv) n += p.second - p.first;
  return n;
}

// Text ranks present after keeping [0, n_sink) and [text_lo, n_text).
std::vector<std::pair<int64_t, int64_t>> iv_after_evict(
    const std::vector<std::pair<int64_t, int64_t>>& iv, int64_t n_sink, int64_t text_lo) {
  if (text_lo <= n_sink) return iv;  // sink and window meet: every text token stays
  std::vector<std::pair<int64_t, int64_t>> out;
  auto push = [&](int64_t a, int64_t b) {
    if (a >= b) return;
    if (!out.empty() && out.back().second == a) out.back().second = b;
    else out.emplace_back(a, b);
  };
  for (auto& p : iv) {
    push(p.first, std::min(p.second, n_sink));
    push(std::max(p.first, text_lo), p.second);
  }
  return out;
}

// Host bookkeeping of n text tokens registered at the end of a stream (the metadata launch is the caller's).
void note_text_registered(sv::StreamState& st, int n, bool cs_tab_valid) {
  st.cs_tab_valid = cs_tab_valid;
  st.pending_slot0 = st.len;
  st.pending_n = n;
  st.next_parity ^= 1;
  st.next_gid += n;
  if (!st.text_iv.empty() && st.text_iv.back().second == st.n_text) st.text_iv.back().second += n;
  else st.text_iv.emplace_back(st.n_text, st.n_text + n);
  st.n_text += n;
  st.len += n;
}

#define SV_HIP(expr)                         \
  do {                                       \
    hipError_t e__ = (expr);                 \
    if (e__ != hipSuccess) return SV_ERR_HIP; \
  } while (0)

// Device work of a call: skipped for a cache created with SV_FLAG_HOST_LOGIC_ONLY.
#define SV_DEV(expr)                 \
  do {                               \
    if (!c->host_logic_only) SV_HIP(expr); \
  } while (0)

}  // namespace

extern "C" {

const char* sv_strerror(int status) {
  switch (status) {
    case SV_OK: return "ok";
    case SV_ERR_INVALID: return "invalid argument";
    case SV_ERR_CAPACITY: return "capacity exceeded";
    case SV_ERR_STATE: return "call order violated";
    case SV_ERR_HIP: return "HIP runtime error";
    case SV_ERR_UNSUPPORTED: return "unsupported configuration";
    default: return "unknown status";
  }
}

size_t sv_cache_bytes(const sv_config* cfg) {
  if (!config_ok(cfg)) return 0;
  return make_layout(*cfg).total;
}

int sv_cache_create(const sv_config* cfg, void* dev_arena, size_t arena_bytes, void* hip_stream,
                    sv_cache** out) {
  if (!out) return SV_ERR_INVALID;
  *out = nullptr;
  if (!config_ok(cfg) || !dev_arena) return SV_ERR_INVALID;
  if (((uintptr_t)dev_arena) % kAlign != 0) return SV_ERR_INVALID;
  Layout L = make_layout(*cfg);
  if (arena_bytes < L.total) return SV_ERR_CAPACITY;
  sv_cache* c = new (std::nothrow) sv_cache();
  if (!c) return SV_ERR_INVALID;
  c->cfg = *cfg;
  c->esize = cfg->dtype == SV_DTYPE_F32 ? 4 : 2;
  c->group = cfg->n_q_heads / cfg->n_kv_heads;
  c->row_bytes = (size_t)cfg->head_dim * c->esize;
  c->cap_pad = (cfg->capacity_tokens + 63) / 64 * 64;
  c->head_stride = (size_t)c->cap_pad * c->row_bytes;
  c->tensor_stride = (size_t)cfg->n_kv_heads * c->head_stride;
  c->layer_stride = 2 * c->tensor_stride;
  c->half_stride = (size_t)cfg->n_layers * c->layer_stride;
  c->stream_kv_stride = 2 * c->half_stride;
  char* base = (char*)dev_arena;
  c->kv_base = base + L.kv;
  for (int h = 0; h < 2; ++h) {
    c->meta[h].gid = (int64_t*)(base + L.meta_gid[h]);
    c->meta[h].rank = (int64_t*)(base + L.meta_rank[h]);
    c->meta[h].pos4 = (int4*)(base + L.meta_pos[h]);
    c->meta[h].local4 = (short4*)(base + L.meta_local[h]);
    c->meta[h].blk = (int32_t*)(base + L.meta_blk[h]);
    c->meta[h].type = (uint8_t*)(base + L.meta_type[h]);
  }
  c->src = (int32_t*)(base + L.src);
  c->delta = (int32_t*)(base + L.delta);
  c->dtab = (float2*)(base + L.dtab);
  c->next_pos = (int32_t*)(base + L.next_pos);
  c->n_dev = (int32_t*)(base + L.n_dev);
  c->inv_freq = (double*)(base + L.inv_freq);
  c->last_cs = (float2*)(base + L.last_cs);
  c->cs_tab = (float2*)(base + L.cs_tab);
  c->part_o = (float*)(base + L.part_o);
  c->part_ml = (float*)(base + L.part_ml);
  c->part_rows = L.part_rows;
  c->counters = (int32_t*)(base + L.counters);
  c->part_dec = (unsigned long long*)(base + L.part_dec);
  c->scan_agg = (unsigned long long*)(base + L.scan_agg);
  c->st.resize(cfg->n_streams);
  for (auto& s : c->st) s.layer_len.assign(cfg->n_layers, 0);
  c->use_mfma = mfma_eligible(*cfg);
  c->v_blocked = c->use_mfma;

  // rotary frequencies theta^(-2i/d), computed once in double
  const int half = cfg->head_dim / 2;
  std::vector<double> f(half, 0.0);
  if (cfg->rope_mode != SV_ROPE_NONE)
    for (int i = 0; i < half; ++i) f[i] = std::pow(cfg->rope_theta, -2.0 * (double)i / (double)cfg->head_dim);
  hipStream_t s = (hipStream_t)hip_stream;
  c->host_logic_only = (cfg->flags & SV_FLAG_HOST_LOGIC_ONLY) != 0;
  if (c->host_logic_only) {   // test seam: bookkeeping and checks only, the arena is never touched
    *out = c;
    return SV_OK;
  }
  hipError_t e = hipMemcpyAsync(c->inv_freq, f.data(), half * sizeof(double), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = hipMemsetAsync(c->next_pos, 0, (size_t)cfg->n_streams * 2 * 4, s);
  if (e == hipSuccess) e = hipMemsetAsync(c->n_dev, 0, (size_t)cfg->n_streams * 4, s);
  if (e == hipSuccess) e = hipMemsetAsync(c->counters, 0, (size_t)L.part_rows * cfg->n_kv_heads * 4, s);
  if (e == hipSuccess && L.part_dec_bytes > 0) e = hipMemsetAsync(c->part_dec, 0, L.part_dec_bytes, s);
  if (e == hipSuccess) e = hipMemsetAsync(c->scan_agg, 0, (size_t)cfg->n_streams * 2 * (sv::kScanMaxWG + 1) * 8, s);
  // blocked V^T: slots past a stream's end inside its last block are multiplied by probabilities of zero and must
  // never hold NaN patterns, so the store starts out cleared
  if (e == hipSuccess && c->v_blocked)
    e = hipMemsetAsync(c->kv_base, 0, (size_t)cfg->n_streams * c->stream_kv_stride, s);
  if (e == hipSuccess && c->use_mfma) e = sv::attn_chunk_mfma_init();
  if (e == hipSuccess && c->use_mfma) {   // device address of sv_attn_decode_static's scratch array, once per device
    void* p = nullptr;
    e = sv::decode_static_scratch(&p);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);  // f is a local: the copy must have read it
  if (e != hipSuccess) {
    delete c;
    return SV_ERR_HIP;
  }
  *out = c;
  return SV_OK;
}

int sv_cache_destroy(sv_cache* c) {
  if (!c) return SV_ERR_INVALID;
  delete c;
  return SV_OK;
}

int sv_cache_set_option(sv_cache* c, int option, int value) {
  if (!c || option < 0 || option >= SV_OPT_COUNT_ || value < 0) return SV_ERR_INVALID;
  c->opt[option] = value;
  return SV_OK;
}

int sv_cache_len(sv_cache* c, int stream_id, int64_t* n_out) {
  if (!stream_ok(c, stream_id) || !n_out) return SV_ERR_INVALID;
  *n_out = c->st[stream_id].len;
  return SV_OK;
}

// sv_cache_append, with the option of leaving the K/V store to the caller (sv_stream_step stores a chunk's K rows and
// V^T blocks and rotates its Q in one launch of its own): all checks and bookkeeping are the same.
static int append_impl(sv_cache* c, int stream_id, int layer, int n, const uint8_t* types_host,
                       const int32_t* grid_thw_host, const void* k_dev, const void* v_dev,
                       int64_t* slot0_out, void* hip_stream, bool launch_kv) {
  if (!stream_ok(c, stream_id) || layer < 0 || layer >= c->cfg.n_layers || n < 0) return SV_ERR_INVALID;
  sv::StreamState& st = c->st[stream_id];
  hipStream_t s = (hipStream_t)hip_stream;
  if (n == 0) {
    if (slot0_out) *slot0_out = st.len;
    return SV_OK;
  }
  if (!k_dev || !v_dev) return SV_ERR_INVALID;

  if (layer == 0) {
    if (!types_host) return SV_ERR_INVALID;
    for (int l = 0; l < c->cfg.n_layers; ++l)
      if (st.layer_len[l] != st.len) return SV_ERR_STATE;  // previous append not finished on every layer
    int n_vis = 0;
    for (int j = 0; j < n; ++j) {
      if (types_host[j] != SV_TEXT && types_host[j] != SV_VISION) return SV_ERR_INVALID;
      n_vis += types_host[j] == SV_VISION;
    }
    int gT = 0, gH = 0, gW = 0;
    if (grid_thw_host) {
      gT = grid_thw_host[0], gH = grid_thw_host[1], gW = grid_thw_host[2];
      if (gT < 1 || gH < 1 || gW < 1 || gT > 32767 || gH > 32767 || gW > 32767) return SV_ERR_INVALID;
      if ((int64_t)gT * gH * gW != n || n_vis != n) return SV_ERR_INVALID;
    } else if (c->cfg.rope_mode == SV_ROPE_3D && n_vis != 0) {
      return SV_ERR_INVALID;  // 3-D positions of vision tokens need their grid
    }
    const int type_uniform = n_vis == 0 ? SV_TEXT : (n_vis == n ? SV_VISION : -1);
    if (type_uniform < 0 && n > sv::kMaxMixedAppend) return SV_ERR_UNSUPPORTED;
    if (st.len + n > c->cfg.capacity_tokens) return SV_ERR_CAPACITY;

    sv::TypeMask mask;
    if (type_uniform < 0) {
      std::memset(&mask, 0, sizeof(mask));
      for (int j = 0; j < n; ++j)
        if (types_host[j] == SV_VISION) mask.w[j >> 5] |= 1u << (j & 31);
    }
    const bool has_blk = grid_thw_host && c->cfg.rope_mode == SV_ROPE_3D;
    // blocked-V^T caches keep the cos/sin of a run of at most max_q_tokens tokens: every layer's K store and, in
    // sv_stream_step, the attention kernel's Q rotation read them instead of evaluating sincos again
    const bool with_cs = c->v_blocked && c->cfg.rope_mode != SV_ROPE_NONE && n <= c->cfg.max_q_tokens;
    SV_DEV(sv::launch_meta_append(c, stream_id, st.next_parity, st.len, n, st.next_gid, st.n_text,
                                  st.n_vis, type_uniform, type_uniform < 0 ? &mask : nullptr,
                                  has_blk ? st.next_blk : -1, gT, gH, gW, with_cs, s));
    st.cs_tab_valid = with_cs;
    st.pending_slot0 = st.len;
    st.pending_n = n;
    if (launch_kv) SV_DEV(sv::launch_append_kv(c, stream_id, 0, st.len, n, k_dev, v_dev, s));

    st.next_parity ^= 1;
    if (has_blk) st.next_blk++;
    st.next_gid += n;
    if (st.len == st.front && st.n_text == st.front)   // the cache is the opening text run so far: it may grow
      for (int j = 0; j < n && types_host[j] == SV_TEXT; ++j) ++st.front;
    const int n_text_new = n - n_vis;
    if (n_text_new > 0) {
      if (!st.text_iv.empty() && st.text_iv.back().second == st.n_text)
        st.text_iv.back().second += n_text_new;
      else
        st.text_iv.emplace_back(st.n_text, st.n_text + n_text_new);
      st.n_text += n_text_new;
    }
    st.n_vis += n_vis;
    st.len += n;
    st.layer_len[0] = st.len;
    if (slot0_out) *slot0_out = st.pending_slot0;
    return SV_OK;
  }

  // layers 1..L-1 repeat the append registered by layer 0
  if (st.layer_len[layer] != st.pending_slot0 || n != st.pending_n ||
      st.pending_slot0 + n != st.len || st.layer_len[0] != st.len)
    return SV_ERR_STATE;
  if (launch_kv) SV_DEV(sv::launch_append_kv(c, stream_id, layer, st.pending_slot0, n, k_dev, v_dev, s));
  st.layer_len[layer] = st.len;
  if (slot0_out) *slot0_out = st.pending_slot0;
  return SV_OK;
}

int sv_cache_append(sv_cache* c, int stream_id, int layer, int n, const uint8_t* types_host,
                    const int32_t* grid_thw_host, const void* k_dev, const void* v_dev,
                    int64_t* slot0_out, void* hip_stream) {
  return append_impl(c, stream_id, layer, n, types_host, grid_thw_host, k_dev, v_dev, slot0_out, hip_stream, true);
}

int sv_cache_evict(sv_cache* c, int stream_id, int64_t n_sink, int64_t vision_window,
                   int64_t text_window, int64_t* n_retained_out, void* hip_stream) {
  if (!stream_ok(c, stream_id)) return SV_ERR_INVALID;
  if (n_sink < 0 || vision_window < SV_WINDOW_INF || text_window < SV_WINDOW_INF) return SV_ERR_INVALID;
  sv::StreamState& st = c->st[stream_id];
  for (int l = 0; l < c->cfg.n_layers; ++l)
    if (st.layer_len[l] != st.len) return SV_ERR_STATE;
  hipStream_t s = (hipStream_t)hip_stream;

  const int64_t kMin = std::numeric_limits<int64_t>::min();
  const int64_t text_lo = text_window == SV_WINDOW_INF ? kMin : st.n_text - std::min(text_window, st.n_text);
  const int64_t vis_lo = vision_window == SV_WINDOW_INF ? kMin : st.n_vis - std::min(vision_window, st.n_vis);

  auto iv_new = iv_after_evict(st.text_iv, n_sink, text_lo);
  const int64_t vis_lo_new = std::max(st.vis_lo, vis_lo);
  const int64_t n_new = iv_count(iv_new) + (st.n_vis - vis_lo_new);
  if (n_retained_out) *n_retained_out = n_new;
  if (n_new == st.len) return SV_OK;  // nothing to evict: no device work

  // The opening text run: its tokens of rank >= n_sink and < text_lo leave; the slots before the first of them
  // (all of the run if none leaves) keep place, position and contents.  What the eviction before this one left in
  // place as well is already in the half this one fills.
  const int64_t gone = (n_sink < st.front && text_lo > n_sink) ? n_sink : st.front;
  const int64_t n_still = std::min(st.still[st.cur], gone);
  SV_DEV(sv::launch_evict_scan(c, stream_id, st.next_parity, st.len, n_sink, text_lo, vis_lo, s));
  if (n_new > 0) SV_DEV(sv::launch_compact(c, stream_id, n_new, n_still, s));
  st.still[st.cur ^ 1] = gone;
  st.front = gone;
  st.cur ^= 1;
  st.next_parity ^= 1;
  st.text_iv.swap(iv_new);
  st.vis_lo = vis_lo_new;
  st.len = n_new;
  for (int l = 0; l < c->cfg.n_layers; ++l) st.layer_len[l] = n_new;
  st.pending_slot0 = n_new;
  st.pending_n = 0;
  st.cs_tab_valid = false;
  return SV_OK;
}

int sv_rope_apply(sv_cache* c, int stream_id, int64_t slot0, int n, void* q_dev_inout,
                  void* k_dev_inout, void* hip_stream) {
  if (!stream_ok(c, stream_id) || n < 0 || slot0 < 0) return SV_ERR_INVALID;
  if (slot0 + n > c->st[stream_id].len) return SV_ERR_INVALID;
  if (n == 0 || c->cfg.rope_mode == SV_ROPE_NONE || (!q_dev_inout && !k_dev_inout)) return SV_OK;
  SV_DEV(sv::launch_rope_apply(c, stream_id, slot0, n, q_dev_inout, k_dev_inout, (hipStream_t)hip_stream));
  return SV_OK;
}

int sv_attn_chunk(sv_cache* c, int stream_id, int layer, const void* q_dev, int n_q, void* o_dev,
                  int causal, void* hip_stream) {
  if (!stream_ok(c, stream_id) || layer < 0 || layer >= c->cfg.n_layers || !q_dev || !o_dev) return SV_ERR_INVALID;
  sv::StreamState& st = c->st[stream_id];
  if (n_q < 1 || n_q > st.len || n_q > c->cfg.max_q_tokens) return SV_ERR_INVALID;
  if (st.layer_len[layer] != st.len) return SV_ERR_STATE;
  hipStream_t s = (hipStream_t)hip_stream;
  if (c->use_mfma) {
    SV_DEV(sv::launch_attn_chunk_mfma(c, stream_id, layer, q_dev, n_q, o_dev, causal, false, s));
    return SV_OK;
  }
  if (!sv::attn_rows_supported(c)) return SV_ERR_UNSUPPORTED;
  SV_DEV(sv::launch_attn_rows_chunk(c, stream_id, layer, q_dev, n_q, o_dev, causal, s));
  return SV_OK;
}

int sv_attn_decode(sv_cache* c, int layer, const int32_t* stream_ids_host, int n_list,
                   const void* q_dev, void* o_dev, void* hip_stream) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers || !stream_ids_host || n_list < 1 || !q_dev || !o_dev)
    return SV_ERR_INVALID;
  if ((int64_t)n_list > c->part_rows) return SV_ERR_INVALID;
  for (int b = 0; b < n_list; ++b) {
    if (!stream_ok(c, stream_ids_host[b])) return SV_ERR_INVALID;
    const sv::StreamState& st = c->st[stream_ids_host[b]];
    if (st.len < 1) return SV_ERR_INVALID;
    if (st.layer_len[layer] != st.len) return SV_ERR_STATE;
  }
  if (c->use_mfma) {
    SV_DEV(sv::launch_attn_decode_mfma(c, layer, stream_ids_host, n_list, 0, q_dev, nullptr, nullptr, o_dev,
                                       (hipStream_t)hip_stream));
    return SV_OK;
  }
  if (!sv::attn_rows_supported(c)) return SV_ERR_UNSUPPORTED;
  SV_DEV(sv::launch_attn_rows_batch(c, layer, stream_ids_host, n_list, 0, q_dev, nullptr, nullptr, o_dev,
                                    (hipStream_t)hip_stream));
  return SV_OK;
}

int sv_attn_decode_static(sv_cache* c, int layer, const int32_t* stream_ids_host, int n_list, const void* q_dev,
                          void* o_dev, void* hip_stream) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers || !stream_ids_host || n_list < 1 || !q_dev || !o_dev)
    return SV_ERR_INVALID;
  if (!c->use_mfma) return SV_ERR_UNSUPPORTED;
  if (n_list > SV_STATIC_MAX_ROWS || (int64_t)n_list > sv::decode_static_pairs(c)) return SV_ERR_CAPACITY;
  for (int b = 0; b < n_list; ++b) {
    if (!stream_ok(c, stream_ids_host[b])) return SV_ERR_INVALID;
    const sv::StreamState& st = c->st[stream_ids_host[b]];
    if (st.len < 1) return SV_ERR_INVALID;
    if (st.layer_len[layer] != st.len) return SV_ERR_STATE;
  }
  SV_DEV(sv::launch_attn_decode_mfma_static(c, layer, stream_ids_host, n_list, q_dev, o_dev, (hipStream_t)hip_stream));
  return SV_OK;
}

int sv_decode_step(sv_cache* c, int layer, const int32_t* stream_ids_host, int n_list, const void* q_dev,
                   const void* k_dev, const void* v_dev, void* o_dev, void* hip_stream) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers || !stream_ids_host || n_list < 1 || !q_dev || !k_dev || !v_dev ||
      !o_dev)
    return SV_ERR_INVALID;
  if ((int64_t)n_list > c->part_rows) return SV_ERR_INVALID;
  const bool use_mfma = c->use_mfma;
  if (!use_mfma && !sv::attn_rows_supported(c)) return SV_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)hip_stream;
  // validate everything before changing anything
  for (int b = 0; b < n_list; ++b) {
    if (!stream_ok(c, stream_ids_host[b])) return SV_ERR_INVALID;
    for (int b2 = 0; b2 < b; ++b2)
      if (stream_ids_host[b2] == stream_ids_host[b]) return SV_ERR_INVALID;  // one new token per stream
    const sv::StreamState& st = c->st[stream_ids_host[b]];
    if (layer == 0) {
      for (int l = 0; l < c->cfg.n_layers; ++l)
        if (st.layer_len[l] != st.len) return SV_ERR_STATE;
      if (st.len + 1 > c->cfg.capacity_tokens) return SV_ERR_CAPACITY;
    } else if (st.layer_len[layer] != st.pending_slot0 || st.pending_n != 1 || st.pending_slot0 + 1 != st.len ||
               st.layer_len[0] != st.len) {
      return SV_ERR_STATE;
    }
  }
  for (int b = 0; b < n_list; ++b) {
    const int sid = stream_ids_host[b];
    sv::StreamState& st = c->st[sid];
    if (layer == 0) {
      SV_DEV(sv::launch_meta_append(c, sid, st.next_parity, st.len, 1, st.next_gid, st.n_text, st.n_vis, SV_TEXT,
                                    nullptr, -1, 0, 0, 0, false, s));
      note_text_registered(st, 1, false);
    }
    st.layer_len[layer] = st.len;
  }
  if (use_mfma) SV_DEV(sv::launch_attn_decode_mfma(c, layer, stream_ids_host, n_list, 1, q_dev, k_dev, v_dev, o_dev, s));
  else SV_DEV(sv::launch_attn_rows_batch(c, layer, stream_ids_host, n_list, 1, q_dev, k_dev, v_dev, o_dev, s));
  return SV_OK;
}

int sv_decode_step_layers(sv_cache* c, int stream_id, const void* q_dev, const void* k_dev, const void* v_dev,
                          void* o_dev, void* hip_stream) {
  if (!stream_ok(c, stream_id) || !q_dev || !k_dev || !v_dev || !o_dev) return SV_ERR_INVALID;
  if (!c->use_mfma) return SV_ERR_UNSUPPORTED;
  const int L = c->cfg.n_layers;
  if ((int64_t)L > c->part_rows) return SV_ERR_INVALID;
  sv::StreamState& st = c->st[stream_id];
  for (int l = 0; l < L; ++l)
    if (st.layer_len[l] != st.len) return SV_ERR_STATE;
  if (st.len + 1 > c->cfg.capacity_tokens) return SV_ERR_CAPACITY;
  hipStream_t s = (hipStream_t)hip_stream;
  SV_DEV(sv::launch_meta_append(c, stream_id, st.next_parity, st.len, 1, st.next_gid, st.n_text, st.n_vis, SV_TEXT,
                                nullptr, -1, 0, 0, 0, false, s));
  note_text_registered(st, 1, false);
  for (int l = 0; l < L; ++l) st.layer_len[l] = st.len;
  const int32_t sid = stream_id;
  SV_DEV(sv::launch_attn_decode_mfma(c, -1, &sid, L, 1, q_dev, k_dev, v_dev, o_dev, s));
  return SV_OK;
}

int sv_stream_step(sv_cache* c, int stream_id, int64_t n_sink, int64_t vision_window, int64_t text_window,
                   const sv_chunk_io* io, int64_t* n_retained_out, void* hip_stream) {
  if (!stream_ok(c, stream_id) || !io || io->n_vision < 0 || io->n_text < 0) return SV_ERR_INVALID;
  if (io->n_vision > 0 && (!io->q_vision || !io->k_vision || !io->v_vision || !io->o_vision)) return SV_ERR_INVALID;
  if (io->n_text > 0 && (!io->q_text || !io->k_text || !io->v_text || !io->o_text)) return SV_ERR_INVALID;
  const int L = c->cfg.n_layers;
  const size_t qrow = (size_t)c->cfg.n_q_heads * c->row_bytes, kvrow = (size_t)c->cfg.n_kv_heads * c->row_bytes;
  int rc = sv_cache_evict(c, stream_id, n_sink, vision_window, text_window, n_retained_out, hip_stream);
  if (rc != SV_OK) return rc;
  if (io->n_vision > 0) {
    const int n = io->n_vision;
    std::vector<uint8_t> types((size_t)n, (uint8_t)SV_VISION);
    const bool has_grid = io->grid_thw[0] > 0 || io->grid_thw[1] > 0 || io->grid_thw[2] > 0;
    // blocked-V^T caches: K/V store and Q rotation of a layer go out as ONE launch
    const bool fused = c->v_blocked && n <= c->cfg.max_q_tokens;
    for (int l = 0; l < L; ++l) {
      int64_t slot0 = 0;
      char* q = (char*)io->q_vision + (size_t)l * n * qrow;
      const char* k = (const char*)io->k_vision + (size_t)l * n * kvrow;
      const char* v = (const char*)io->v_vision + (size_t)l * n * kvrow;
      char* o = (char*)io->o_vision + (size_t)l * n * qrow;
      rc = append_impl(c, stream_id, l, n, types.data(), has_grid ? io->grid_thw : nullptr, k, v, &slot0, hip_stream,
                       !fused);
      if (rc != SV_OK) return rc;
      if (fused) {
        // Q stays as the caller wrote it when the run's cos/sin table exists and few key ranges will load each query
        // row: the attention kernel then rotates it on load
        // ... and a short chunk's K/V are stored by the attention launch itself
        if (st_cs_valid(c, stream_id) && sv::attn_chunk_stores_tokens(c, stream_id, n)) {
          SV_DEV(sv::launch_attn_chunk_mfma(c, stream_id, l, q, n, o, 1, true, (hipStream_t)hip_stream, k, v));
          continue;
        }
        const bool q_on_load = st_cs_valid(c, stream_id) && sv::attn_chunk_rotates_on_load(c, stream_id, n);
        SV_DEV(sv::launch_store_tokens_vt(c, stream_id, l, slot0, n, q_on_load ? nullptr : q, k, v,
                                          (hipStream_t)hip_stream));
        SV_DEV(sv::launch_attn_chunk_mfma(c, stream_id, l, q, n, o, 1, q_on_load, (hipStream_t)hip_stream));
      } else {
        rc = sv_rope_apply(c, stream_id, slot0, n, q, nullptr, hip_stream);
        if (rc != SV_OK) return rc;
        rc = sv_attn_chunk(c, stream_id, l, q, n, o, 1, hip_stream);
        if (rc != SV_OK) return rc;
      }
    }
  }
  const int32_t sid = stream_id;
  if (io->decode_layers_batched) {
    for (int t = 0; t < io->n_text; ++t) {
      const size_t i = (size_t)t * L;
      rc = sv_decode_step_layers(c, stream_id, (const char*)io->q_text + i * qrow, (const char*)io->k_text + i * kvrow,
                                 (const char*)io->v_text + i * kvrow, (char*)io->o_text + i * qrow, hip_stream);
      if (rc != SV_OK) return rc;
    }
    return SV_OK;
  }
  if (c->use_mfma && io->n_text > 1 && io->n_text <= c->cfg.max_q_tokens) {
    // The call names its n_text decode steps in advance, and what a decoded text token's registration writes (arrival
    // id, rank, position, rotary cos/sin) does not depend on the token: the run is registered ONCE, as an append of
    // n_text text tokens whose K/V arrive later, and the fused decode launch of step t stores token t and attends to
    // the first len0 + t + 1 slots with the cos/sin row t of the run's table.  Same result as n_text single-token
    // registrations (the table holds what each of them would have computed), n_text - 1 launches fewer.
    sv::StreamState& st = c->st[stream_id];
    const int n = io->n_text;
    for (int l = 0; l < L; ++l)
      if (st.layer_len[l] != st.len) return SV_ERR_STATE;
    if (st.len + n > c->cfg.capacity_tokens) return SV_ERR_CAPACITY;
    const int64_t len0 = st.len;
    const bool with_cs = c->cfg.rope_mode != SV_ROPE_NONE;
    SV_DEV(sv::launch_meta_append(c, stream_id, st.next_parity, len0, n, st.next_gid, st.n_text, st.n_vis, SV_TEXT, nullptr,
                                  -1, 0, 0, 0, with_cs, (hipStream_t)hip_stream));
    note_text_registered(st, n, with_cs);
    for (int t = 0; t < n; ++t)
      for (int l = 0; l < L; ++l) {
        const size_t i = (size_t)t * L + l;
        SV_DEV(sv::launch_decode_step_of_run(c, l, stream_id, len0 + t + 1, t, (const char*)io->q_text + i * qrow,
                                             (const char*)io->k_text + i * kvrow, (const char*)io->v_text + i * kvrow,
                                             (char*)io->o_text + i * qrow, (hipStream_t)hip_stream));
      }
    for (int l = 0; l < L; ++l) st.layer_len[l] = st.len;
    return SV_OK;
  }
  for (int t = 0; t < io->n_text; ++t)
    for (int l = 0; l < L; ++l) {
      const size_t i = (size_t)t * L + l;
      rc = sv_decode_step(c, l, &sid, 1, (const char*)io->q_text + i * qrow, (const char*)io->k_text + i * kvrow,
                          (const char*)io->v_text + i * kvrow, (char*)io->o_text + i * qrow, hip_stream);
      if (rc != SV_OK) return rc;
    }
  return SV_OK;
}

int sv_cache_retained(sv_cache* c, int stream_id, int64_t* ids_host, int32_t* pos3_host, int64_t cap,
                      int64_t* n_out, void* hip_stream) {
  if (!stream_ok(c, stream_id) || cap < 0) return SV_ERR_INVALID;
  sv::StreamState& st = c->st[stream_id];
  hipStream_t s = (hipStream_t)hip_stream;
  if (n_out) *n_out = st.len;
  if (c->host_logic_only) return SV_ERR_UNSUPPORTED;   // ids and positions live in device memory
  const int64_t n = std::min(cap, st.len);
  const size_t off = (size_t)stream_id * (size_t)c->cfg.capacity_tokens;
  std::vector<int4> pos;
  int32_t n_dev = -1;   // the device's own count: written by the eviction scan and by every registration
  SV_HIP(hipMemcpyAsync(&n_dev, c->n_dev + stream_id, 4, hipMemcpyDeviceToHost, s));
  if (n > 0 && ids_host)
    SV_HIP(hipMemcpyAsync(ids_host, c->meta[st.cur].gid + off, (size_t)n * 8, hipMemcpyDeviceToHost, s));
  if (n > 0 && pos3_host) {
    pos.resize(n);
    SV_HIP(hipMemcpyAsync(pos.data(), c->meta[st.cur].pos4 + off, (size_t)n * 16, hipMemcpyDeviceToHost, s));
  }
  SV_HIP(hipStreamSynchronize(s));
  if ((int64_t)n_dev != st.len) return SV_ERR_STATE;   // host bookkeeping and device scan disagree
  if (n > 0 && pos3_host)
    for (int64_t i = 0; i < n; ++i) {
      pos3_host[3 * i + 0] = pos[i].x;
      pos3_host[3 * i + 1] = pos[i].y;
      pos3_host[3 * i + 2] = pos[i].z;
    }
  return SV_OK;
}

int sv_cache_read_kv(sv_cache* c, int stream_id, int layer, int which, int64_t slot0, int64_t n,
                     void* dst_host, void* hip_stream) {
  if (!stream_ok(c, stream_id) || layer < 0 || layer >= c->cfg.n_layers || (which != 0 && which != 1))
    return SV_ERR_INVALID;
  sv::StreamState& st = c->st[stream_id];
  if (slot0 < 0 || n < 0 || slot0 + n > st.layer_len[layer] || (n > 0 && !dst_host)) return SV_ERR_INVALID;
  if (c->host_logic_only) return SV_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)hip_stream;
  if (n > 0 && which == 1 && c->v_blocked) {
    // blocked V^T: fetch the 8-key blocks that cover the rows and pick the elements out on the host
    const int64_t b0 = slot0 / sv::kVB, nb = (slot0 + n - 1) / sv::kVB - b0 + 1;
    std::vector<uint16_t> tmp((size_t)c->cfg.n_kv_heads * nb * sv::kVBElems);
    for (int h = 0; h < c->cfg.n_kv_heads; ++h)
      SV_HIP(hipMemcpyAsync(tmp.data() + (size_t)h * nb * sv::kVBElems,
                            c->kv_ptr(stream_id, st.cur, layer, 1) + (size_t)h * c->head_stride + (size_t)b0 * sv::kVBElems * 2,
                            (size_t)nb * sv::kVBElems * 2, hipMemcpyDeviceToHost, s));
    SV_HIP(hipStreamSynchronize(s));
    uint16_t* dst = (uint16_t*)dst_host;
    for (int64_t i = 0; i < n; ++i)
      for (int h = 0; h < c->cfg.n_kv_heads; ++h)
        for (int d = 0; d < c->cfg.head_dim; ++d)
          dst[((size_t)i * c->cfg.n_kv_heads + h) * c->cfg.head_dim + d] =
              tmp[(size_t)h * nb * sv::kVBElems + sv::vt_elem(slot0 + i - b0 * sv::kVB, d)];
    return SV_OK;
  }
  if (n > 0) {
    const char* src = c->kv_ptr(stream_id, st.cur, layer, which) + (size_t)slot0 * c->row_bytes;
    const size_t dpitch = (size_t)c->cfg.n_kv_heads * c->row_bytes;
    for (int h = 0; h < c->cfg.n_kv_heads; ++h)
      SV_HIP(hipMemcpy2DAsync((char*)dst_host + (size_t)h * c->row_bytes, dpitch,
                              src + (size_t)h * c->head_stride, c->row_bytes, c->row_bytes, (size_t)n,
                              hipMemcpyDeviceToHost, s));
  }
  SV_HIP(hipStreamSynchronize(s));
  return SV_OK;
}

}  // extern "C"
