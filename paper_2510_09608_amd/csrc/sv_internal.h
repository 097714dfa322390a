// Internal declarations shared by the host side of libsv and its kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "sv.h"

namespace sv {

// ---- blocked V^T layout (caches with v_blocked: bf16, head_dim 128, matrix-core kernels) -----------------
// Both attention kernels contract V over keys, so their matrix-core operand is a piece of V^T: one head dim,
// 8 consecutive keys per lane.  V is therefore STORED transposed in blocks of kVB = 8 keys: per kv head, block b
// holds keys [8 b, 8 b + 8) as [head dim 0..127][key 0..7] (2 KB), element (key, d) at vt_elem(key, d).  A block
// row is exactly the 16-byte piece a lane wants; 32- and 64-key tiles are 4 and 8 consecutive blocks (8 / 16 KB
// contiguous); and a compaction that drops runs of 8 k tokens moves whole blocks.
constexpr int kScanMaxWG = 128;   // workgroups of one eviction scan
constexpr int kVB = 8;
constexpr int kVD = 128;
constexpr int kVBElems = kVB * kVD;
__host__ __device__ inline size_t vt_elem(int64_t key, int d) {
  return (size_t)(key >> 3) * kVBElems + (size_t)d * kVB + (size_t)(key & 7);
}

// ---- per-token metadata kept in device memory, structure of arrays -----------------
// pos4  : (t, h, w, base).  base is the scalar position the token's block starts at
//         (for text and for 1-D mode it equals t); the shift applied by an eviction
//         is old base - new base and is common to t, h and w.
// local4: (lt, lh, lw, extent) of a vision token inside its block; text is (0,0,0,1).
// blk   : vision block id, -1 for text and for vision tokens appended without a grid.
struct MetaPtrs {
  int64_t* gid;
  int64_t* rank;
  int4* pos4;
  short4* local4;
  int32_t* blk;
  uint8_t* type;
};

struct StreamState {
  int64_t len = 0;        // tokens in cache
  int64_t n_text = 0;     // text tokens ever appended
  int64_t n_vis = 0;      // vision tokens ever appended
  int64_t next_gid = 0;
  int32_t next_blk = 0;
  int cur = 0;            // which half of the ping-pong store is live
  int next_parity = 0;    // which entry of next_pos[stream][2] is live
  int64_t vis_lo = 0;     // vision ranks present are [vis_lo, n_vis)
  std::vector<std::pair<int64_t, int64_t>> text_iv;  // text ranks present, disjoint half-open intervals
  std::vector<int64_t> layer_len;                    // tokens stored per layer
  int64_t pending_slot0 = 0;                         // first slot of the append in flight
  int pending_n = 0;
  bool cs_tab_valid = false;                         // cs_tab holds the rotary cos/sin of the pending run's tokens
  // Slots [0, front) hold the text tokens of rank 0 .. front - 1: the stream's opening text run (system prompt and
  // what follows it before the first vision token), as far as evictions have left it in place.  An eviction leaves
  // the slots below the run's first leaving token where they are, unshifted; still[h] is that bound for the eviction
  // that filled K/V half h, so below min(still[0], still[1]) both halves hold the same rows and the next eviction
  // need not move them again.
  int64_t front = 0;
  int64_t still[2] = {0, 0};
};

}  // namespace sv

struct sv_cache {
  sv_config cfg;
  int esize;                 // bytes per element
  int group;                 // q heads per kv head
  size_t row_bytes;          // head_dim * esize
  int64_t cap_pad;           // capacity rounded up to 64 slots
  size_t head_stride;        // cap_pad * row_bytes            (one kv head of one tensor)
  size_t tensor_stride;      // n_kv_heads * head_stride       (K or V of one layer)
  size_t layer_stride;       // 2 * tensor_stride
  size_t half_stride;        // n_layers * layer_stride        (one ping-pong half)
  size_t stream_kv_stride;   // 2 * half_stride
  char* kv_base;             // device
  sv::MetaPtrs meta[2];      // device, stream 0; per-stream offset = stream * capacity elements
  int32_t* src;              // device [n_streams][capacity]   gather list of the last eviction
  int32_t* delta;            // device [n_streams][capacity]   position shift of the last eviction
  float2* dtab;              // device [n_streams][capacity][head_dim/2]  cos/sin of the shift
  int32_t* next_pos;         // device [n_streams][2]          scalar position of the next token (ping-pong)
  int32_t* n_dev;            // device [n_streams]             retained count written by the scan
  double* inv_freq;          // device [head_dim/2]
  float2* last_cs;           // device [n_streams][head_dim/2]  cos/sin at the position of the newest token
  float2* cs_tab;            // device [n_streams][max_q_tokens][head_dim/2]  cos/sin of the tokens of the last
                             // registered run (written when it has at most max_q_tokens tokens; blocked-V^T caches)
  float* part_o;             // device split-KV partial outputs
  float* part_ml;            // device split-KV partial (max, sum)
  int64_t part_rows;         // capacity of the partial buffers in (token, split) pairs
  int32_t* counters;         // device [part_rows][n_kv_heads]  arrival counters of the split-KV merge (zero between launches)
  unsigned long long* part_dec;   // device: marked partial results of a single stream's key ranges in the matrix-core
                                  // decode kernel (zero at create and between launches; sv_attn_decode.hip)
  unsigned long long* scan_agg;   // device [n_streams][kScanMaxWG + 1][2]: tagged totals of the eviction scan's
                                  // workgroups, then the scan's launch tag (zero at create, written by nothing else;
                                  // sv_meta.hip)
  bool host_logic_only = false;   // created with SV_FLAG_HOST_LOGIC_ONLY: no device work, bookkeeping only
  bool use_mfma = false;          // bf16, head_dim 128, group <= 8 and no SV_FLAG_GENERIC_KERNELS: matrix-core kernels
  bool v_blocked = false;         // V stored as V^T in blocks of 8 keys (exactly the caches with use_mfma), else row-major
  int opt[SV_OPT_COUNT_] = {};    // sv_cache_set_option values, 0 = automatic
  std::vector<sv::StreamState> st;

  char* kv_ptr(int stream, int half, int layer, int which) const {
    return kv_base + (size_t)stream * stream_kv_stride + (size_t)half * half_stride +
           (size_t)layer * layer_stride + (size_t)which * tensor_stride;
  }
};

namespace sv {

// Kernel launchers (one translation unit each).  All are asynchronous on `s`
// and return the hipError_t of the launch.

// Types of the tokens of one append as a bit mask (bit j set = vision), passed by value.
constexpr int kMaxMixedAppend = 2048;
struct TypeMask {
  uint32_t w[kMaxMixedAppend / 32];
};

// type_uniform: SV_TEXT / SV_VISION when all n tokens share it, -1 to read `mask`.
// with_cs_tab: also write the rotary cos/sin of the n tokens to c->cs_tab (n <= max_q_tokens).
hipError_t launch_meta_append(const sv_cache* c, int stream, int next_parity, int64_t slot0, int n,
                              int64_t gid0, int64_t rank_text0, int64_t rank_vis0, int type_uniform,
                              const TypeMask* mask, int blk, int gT, int gH, int gW, bool with_cs_tab, hipStream_t s);

hipError_t launch_append_kv(const sv_cache* c, int stream, int layer, int64_t slot0, int n,
                            const void* k, const void* v, hipStream_t s);

// Keep rule: text rank < n_sink or rank >= text_lo; vision rank >= vis_lo.
hipError_t launch_evict_scan(const sv_cache* c, int stream, int next_parity, int64_t n_old,
                             int64_t n_sink, int64_t text_lo, int64_t vis_lo, hipStream_t s);

// Slots below `n_still` (rounded down to the kernel's token group) are not moved: the caller knows that the other half
// already holds them.
hipError_t launch_compact(const sv_cache* c, int stream, int64_t n_new, int64_t n_still, hipStream_t s);

hipError_t launch_rope_apply(const sv_cache* c, int stream, int64_t slot0, int n, void* q, void* k,
                             hipStream_t s);

hipError_t launch_attn_rows_chunk(const sv_cache* c, int stream, int layer, const void* q, int n_q,
                                  void* o, int causal, hipStream_t s);
// fused != 0: q is un-rotated and k_new / v_new ([n_list][n_kv_heads][head_dim], un-rotated K) are the
// newest token of each stream, already counted in the stream's length: the kernel rotates q and k_new at
// that token's position and stores k_new / v_new in the cache before attending.
hipError_t launch_attn_rows_batch(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused,
                                  const void* q, const void* k_new, const void* v_new, void* o, hipStream_t s);
bool attn_rows_supported(const sv_cache* c);

// Same contract as launch_attn_rows_batch, matrix-core kernel (c->use_mfma).
hipError_t launch_attn_decode_mfma(const sv_cache* c, int layer, const int32_t* streams, int n_list, int fused,
                                   const void* q, const void* k_new, const void* v_new, void* o, hipStream_t s);

// One fused decode step (append + RoPE + attention) for token `run_index` of the stream's last registered run, whose
// metadata and cos/sin table (c->cs_tab) were written for the whole run at once: the token is slot len - 1, the keys
// are [0, len).
hipError_t launch_decode_step_of_run(const sv_cache* c, int layer, int stream, int64_t len, int run_index, const void* q,
                                     const void* k_new, const void* v_new, void* o, hipStream_t s);

// sv_attn_decode_static: split-KV partials in a file-scope device array instead of the arena.
// decode_static_scratch looks the array's device address up (once per device, kept); decode_static_pairs is the
// number of (row, key range) pairs the array holds for this cache's head count.
hipError_t decode_static_scratch(void** ptr_out);
int64_t decode_static_pairs(const sv_cache* c);
size_t decode_marked_bytes(const sv_config& cfg);   // bytes of sv_cache::part_dec
hipError_t launch_attn_decode_mfma_static(const sv_cache* c, int layer, const int32_t* streams, int n_list,
                                          const void* q, void* o, hipStream_t s);

// Once per process and device, before the first chunk-prefill launch: the kernel's LDS size has to be asked for.
hipError_t attn_chunk_mfma_init();
// Caches with blocked V^T (c->v_blocked): store n new tokens of one layer (K rows rotated, V transposed into its
// blocks) and, if q is not NULL, rotate their Q rows in place, all in one launch.  K takes its cos/sin from
// c->cs_tab when the stream's table is valid for this run.
hipError_t launch_store_tokens_vt(const sv_cache* c, int stream, int layer, int64_t slot0, int n, void* q, const void* k,
                                  const void* v, hipStream_t s);
// rotate_q: q is un-rotated; the kernel rotates it while loading, with c->cs_tab (the queries must be the run the
// table was written for).
// k_new / v_new not NULL (then rotate_q must be set): the n_q tokens are counted in the stream's length and
// registered, but their K/V ([n_q][n_kv_heads][head_dim], K un-rotated) are not in the cache yet: the launch stores
// them (what launch_store_tokens_vt would have) before it reads them.
hipError_t launch_attn_chunk_mfma(const sv_cache* c, int stream, int layer, const void* q, int n_q,
                                  void* o, int causal, bool rotate_q, hipStream_t s, const void* k_new = nullptr,
                                  const void* v_new = nullptr);
// Whether that pays for a chunk of n_q tokens already counted in the stream's length (it does when the workgroups
// that would store have less attention work than the others).
bool attn_chunk_stores_tokens(const sv_cache* c, int stream, int n_q);
// Whether a chunk of n_q queries (already counted in the stream's length) is better rotated by the attention kernel
// while loading than by a pass over Q in memory.
bool attn_chunk_rotates_on_load(const sv_cache* c, int stream, int n_q);


}  // namespace sv
