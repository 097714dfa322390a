/*
 * libsv -- streaming KV-cache hot path of StreamingVLM (arXiv 2510.09608) for
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * One cache object holds, for each of n_streams independent streams and each
 * layer, the K and V rows of the tokens that the streaming policy still
 * retains, in arrival order, in device memory that the CALLER allocates and
 * owns (one arena, see sv_cache_bytes).  The library owns only the opaque
 * handle and a little host bookkeeping, and never allocates device memory.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *     host memory.  Borrowed for the duration of the call, never retained.
 *   - Every device-touching call is asynchronous on the HIP stream passed as
 *     `hip_stream` (a hipStream_t, NULL = default stream); all calls on one
 *     handle must use streams that are ordered with respect to each other.
 *   - All functions return SV_OK (0) or a negative sv_status; nothing throws
 *     or aborts across the boundary.  Host-side outputs (slot numbers, counts)
 *     are valid on return; device outputs after the stream reaches them.
 *   - A handle is not thread-safe; separate handles are independent.
 *   - Token rows: Q is [n][n_q_heads][head_dim], K and V are
 *     [n][n_kv_heads][head_dim], contiguous, in the cache dtype.
 *   - Query head h reads kv head h / (n_q_heads / n_kv_heads); scores are
 *     scaled by 1/sqrt(head_dim); softmax is accumulated in fp32.
 */
#ifndef SV_H_
#define SV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SV_API __attribute__((visibility("default")))

typedef enum sv_status {
  SV_OK = 0,
  SV_ERR_INVALID = -1,     /* bad argument: NULL, out of range, inconsistent shapes   */
  SV_ERR_CAPACITY = -2,    /* append beyond capacity_tokens, or arena too small       */
  SV_ERR_STATE = -3,       /* call order violated (layers not all appended, ...)      */
  SV_ERR_HIP = -4,         /* a HIP runtime call or kernel launch failed              */
  SV_ERR_UNSUPPORTED = -5  /* legal request this build has no kernel for              */
} sv_status;

enum { SV_DTYPE_F32 = 0, SV_DTYPE_BF16 = 1 };
enum { SV_ROPE_1D = 0, SV_ROPE_3D = 1, SV_ROPE_NONE = 2 };
enum { SV_TEXT = 0, SV_VISION = 1 };

/* Budgets equal to SV_WINDOW_INF keep every token of that class (the paper's
 * "infinity" rows in the sink/window ablation, Table 5). */
#define SV_WINDOW_INF (-1)

typedef struct sv_config {
  int32_t n_layers;          /* >= 1                                                   */
  int32_t n_q_heads;         /* multiple of n_kv_heads                                 */
  int32_t n_kv_heads;
  int32_t head_dim;          /* 64 or 128                                              */
  int32_t dtype;             /* SV_DTYPE_*: storage type of Q, K, V and O              */
  int32_t rope_mode;         /* SV_ROPE_*                                              */
  double rope_theta;         /* rotary base; frequency i is theta^(-2i/head_dim)       */
  int32_t mrope_sections[3]; /* SV_ROPE_3D: frequencies read t, then h, then w; sum = head_dim/2 */
  int32_t n_streams;         /* independent streams held by this cache, >= 1           */
  int64_t capacity_tokens;   /* slots per stream                                       */
  int32_t max_q_tokens;      /* largest n_q given to sv_attn_chunk (sizes its scratch) */
  int32_t flags;             /* SV_FLAG_* bits, 0 = default                             */
} sv_config;

/* sv_config.flags.  SV_FLAG_GENERIC_KERNELS: run the generic (vector ALU) attention kernels and keep
 * the row-major V layout even where the matrix-core kernels apply (bf16, head_dim 128, at most 8 query
 * heads per kv head).  Same results to rounding; the parity tests use it to cover the generic kernels
 * on bf16 data.
 * SV_FLAG_HOST_LOGIC_ONLY: a test seam.  The cache launches nothing and never touches the arena: argument
 * checks, call-order rules, lengths, retained counts and error codes behave as usual (they are host
 * bookkeeping), attention outputs are not produced, and sv_cache_retained / sv_cache_read_kv return
 * SV_ERR_UNSUPPORTED.  It exists so that the host logic can be tested on a machine without a GPU. */
enum { SV_FLAG_GENERIC_KERNELS = 1, SV_FLAG_HOST_LOGIC_ONLY = 2 };

typedef struct sv_cache sv_cache;

/* Text for a status code; never NULL. */
SV_API const char* sv_strerror(int status);

/* Bytes of device memory sv_cache_create needs for this configuration (both
 * halves of the ping-pong K/V store, per-token metadata, split-KV scratch).
 * Returns 0 if the configuration is invalid. */
SV_API size_t sv_cache_bytes(const sv_config* cfg);

/* Create a cache inside caller-owned device memory `dev_arena` (256-byte
 * aligned, at least sv_cache_bytes(cfg) bytes, must outlive the handle).  The
 * arena's contents need no initialisation.  Synchronous and cheap: touches the
 * device only to zero a few counters on `hip_stream`.
 * Errors: SV_ERR_INVALID (NULLs, n_q_heads % n_kv_heads, head_dim not 64/128,
 * sections not summing to head_dim/2, sizes < 1, capacity_tokens above 2^24, unknown flag bits),
 * SV_ERR_CAPACITY (arena too small).
 * The library reads no environment variable, here or on any launch path.
 */
SV_API int sv_cache_create(const sv_config* cfg, void* dev_arena, size_t arena_bytes,
                    void* hip_stream, sv_cache** out);

/* Free the handle (host memory only; the arena stays with the caller). */
SV_API int sv_cache_destroy(sv_cache* c);

/*
 * sv_cache_set_option -- per-handle launch overrides; implements no passage of the paper.  Every option
 * defaults to 0 = "let the library choose" (what all measurements use); a positive value forces
 *   SV_OPT_CHUNK_SPLITS           the number of key ranges of sv_attn_chunk's matrix-core kernel,
 *   SV_OPT_DECODE_TILES_PER_WAVE  the 32-key tiles each wavefront of the decode kernel takes (1..16),
 *   SV_OPT_DECODE_SPLITS          the number of key ranges of the generic row kernel,
 *   SV_OPT_CHUNK_STORE            who stores a chunk's K/V in sv_stream_step on a matrix-core cache: 1 = always a
 *                                 launch of its own, 2 = the attention launch whenever it can (chunks of at most
 *                                 512 tokens with a rotary mode); 0 = whichever the library expects to be faster.
 * Forced values are still clamped to what the scratch buffers hold.  Host-side state only: takes effect
 * from the next launch.  Errors: SV_ERR_INVALID (NULL handle, unknown option, negative value).
 */
enum {
  SV_OPT_CHUNK_SPLITS = 0,
  SV_OPT_DECODE_TILES_PER_WAVE = 1,
  SV_OPT_DECODE_SPLITS = 2,
  SV_OPT_CHUNK_STORE = 3,
  SV_OPT_COUNT_ = 4
};
SV_API int sv_cache_set_option(sv_cache* c, int option, int value);

/*
 * sv_cache_append -- new tokens join the cache in arrival order and their K/V
 * states are stored for reuse (Sec. 2.1, "Streaming-aware KV Cache").
 *
 * Appends n tokens to `stream_id` for one `layer`.  The call with layer == 0
 * registers the tokens: it assigns slots [slot0, slot0+n), arrival ids, ranks
 * within their type and contiguous rotary positions that continue from the
 * last retained token (Sec. 2.1, "Contiguous RoPE").  Calls for layers
 * 1..n_layers-1 must follow, in any order, with the same n, before attention
 * on that layer, before the next layer-0 append and before sv_cache_evict
 * (else SV_ERR_STATE).
 *
 *   types_host    [n] SV_TEXT / SV_VISION; read only when layer == 0.
 *   grid_thw_host NULL, or the (T, H, W) grid of one vision block: then every
 *                 type must be SV_VISION and n == T*H*W, tokens in row-major
 *                 (t, h, w) order.  SV_ROPE_3D requires a grid for vision
 *                 tokens and builds their (t, h, w) indices from it; afterwards
 *                 the scalar position advances by max(T, H, W).  Each of T, H,
 *                 W must be <= 32767.
 *   k_dev, v_dev  [n][n_kv_heads][head_dim], K NOT yet rotated: the library
 *                 rotates K at the assigned positions while storing it.
 *   slot0_out     host, optional: first slot assigned.
 * Errors: SV_ERR_CAPACITY when len + n > capacity_tokens (nothing is changed).
 */
SV_API int sv_cache_append(sv_cache* c, int stream_id, int layer, int n,
                    const uint8_t* types_host, const int32_t* grid_thw_host,
                    const void* k_dev, const void* v_dev, int64_t* slot0_out,
                    void* hip_stream);

/*
 * sv_cache_evict -- cut one stream's cache to the three budgets of Sec. 2.1 /
 * Fig. 3 and make it compact again.  A text token stays if it is among the
 * first n_sink text tokens ever appended to the stream or among the last
 * text_window text tokens; a vision token stays if it is among the last
 * vision_window vision tokens.  "First" and "last" go by rank among the tokens of that type EVER
 * appended to the stream (evicted ones included), at the time of the call: with fixed budgets, evicting at
 * every step retains exactly what one eviction at the end would.
 * Survivors keep their order; their K/V rows of all layers are moved to the
 * front (stream compaction), they get new contiguous positions (1-D: the slot
 * index; 3-D: re-walk of the retained list with the block rule, see
 * sv_cache_append), and cached K is re-rotated by the position shift, which
 * is one scalar per token.  Budgets are in tokens; SV_WINDOW_INF for a window
 * keeps the whole class; 0 is legal.  A call that evicts nothing does no
 * device work.  n_retained_out (host, optional) is valid on return.
 * Errors: SV_ERR_STATE if some layer has not received the last append.
 */
SV_API int sv_cache_evict(sv_cache* c, int stream_id, int64_t n_sink, int64_t vision_window,
                   int64_t text_window, int64_t* n_retained_out, void* hip_stream);

/*
 * sv_rope_apply -- rotate fresh Q (and, for callers that keep their own K
 * copies, K) in place at the contiguous positions of cache slots
 * [slot0, slot0+n) of `stream_id` (Sec. 2.1, "Contiguous RoPE": 1-D index, or
 * the 3-D (t, h, w) index where frequency i reads t, h or w by section).
 * Pairing is (i, i + head_dim/2).  q_dev_inout is [n][n_q_heads][head_dim] or
 * NULL; k_dev_inout is [n][n_kv_heads][head_dim] or NULL.  The slots must
 * exist.  With SV_ROPE_NONE this is a no-op.
 */
SV_API int sv_rope_apply(sv_cache* c, int stream_id, int64_t slot0, int n,
                  void* q_dev_inout, void* k_dev_inout, void* hip_stream);

/*
 * sv_attn_chunk -- chunked prefill: the n_q newest tokens of the stream (the
 * last n_q slots, K/V already appended for `layer`) attend to the retained
 * cache and, causally, to their own chunk (Sec. 2.1: new frames reuse the
 * retained states instead of recomputing them).  q_dev is rotated Q
 * [n_q][n_q_heads][head_dim]; o_dev receives [n_q][n_q_heads][head_dim].
 * causal != 0: query i sees slots <= its own; causal == 0: all slots.
 * n_q <= max_q_tokens.
 */
SV_API int sv_attn_chunk(sv_cache* c, int stream_id, int layer, const void* q_dev, int n_q,
                  void* o_dev, int causal, void* hip_stream);

/*
 * sv_attn_decode -- one rotated query token per listed stream attends to that
 * stream's whole cache for `layer`, the newest token (itself) included
 * (text decoding against the compact cache, Sec. 2.1 / Sec. 3.3).  Streams may
 * have different lengths (split-KV, variable length).  q_dev and o_dev are
 * [n_list][n_q_heads][head_dim], row b belongs to stream_ids_host[b].
 */
SV_API int sv_attn_decode(sv_cache* c, int layer, const int32_t* stream_ids_host, int n_list,
                   const void* q_dev, void* o_dev, void* hip_stream);

/*
 * sv_attn_decode_static -- sv_attn_decode for callers that cannot allocate or hand over scratch memory
 * (code under HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments,
 * same result; the partial results of the key ranges go to a fixed 8 MiB device array inside the library
 * (static storage, one copy per GPU, held until the process ends) instead of the arena's scratch region,
 * and the call allocates nothing, on the host or on the device.  Limits: bf16 / head_dim 128 / at most 8
 * query heads per kv head (else SV_ERR_UNSUPPORTED); n_list <= SV_STATIC_MAX_ROWS and
 * n_list * n_q_heads * 516 bytes <= 4 MiB (else SV_ERR_CAPACITY); rows longer than the array's share are
 * cut into fewer, longer key ranges.  Every call on one GPU shares the array: calls that overlap in time on
 * one GPU (different streams, different handles) race; calls ordered on one stream do not.  The array is
 * zero when the library is loaded and needs no clearing between calls: half of it holds the plain partial
 * results of multi-row calls, every entry of which a call writes before its merge launch reads it; the other
 * half holds those of one-row calls as 64-bit words {value, launch tag}, which the call's own workgroups read
 * until they carry the tag of this launch; the tag is kept in the array itself and moved on by every launch.
 * Nothing in a launch depends on host state that changes from call to call, so a captured call may be replayed
 * while the cache is unchanged.
 */
#define SV_STATIC_MAX_ROWS 64
SV_API int sv_attn_decode_static(sv_cache* c, int layer, const int32_t* stream_ids_host, int n_list,
                                 const void* q_dev, void* o_dev, void* hip_stream);

/*
 * sv_decode_step -- one decoded text token per listed stream in a single
 * launch per layer: equivalent to sv_cache_append (one SV_TEXT token),
 * sv_rope_apply on the query and sv_attn_decode, fused (Sec. 2.1: the new
 * token's state joins the cache, gets the next contiguous position, and its
 * query attends to everything retained, itself included).  q_dev
 * [n_list][n_q_heads][head_dim] and k_dev, v_dev [n_list][n_kv_heads][head_dim]
 * are UN-rotated and are not modified; o_dev receives
 * [n_list][n_q_heads][head_dim].  Layer order rules are those of
 * sv_cache_append (layer 0 registers the token).  Streams must be distinct.
 */
SV_API int sv_decode_step(sv_cache* c, int layer, const int32_t* stream_ids_host, int n_list,
                          const void* q_dev, const void* k_dev, const void* v_dev, void* o_dev,
                          void* hip_stream);

/*
 * sv_decode_step_layers -- sv_decode_step of ONE stream for ALL layers in a
 * single launch: layer l is one row of a batched variable-length decode, with
 * q_dev [n_layers][n_q_heads][head_dim], k_dev / v_dev
 * [n_layers][n_kv_heads][head_dim] (un-rotated, not modified) and o_dev
 * [n_layers][n_q_heads][head_dim].  Same result as n_layers calls of
 * sv_decode_step (Sec. 2.1), and only usable where every layer's query exists
 * before any layer's attention runs: attention-only measurement, as here, or a
 * model with parallel layers; a sequential transformer produces layer l + 1's
 * query from layer l's output and has to call sv_decode_step layer by layer.
 * Errors: as sv_decode_step at layer 0; SV_ERR_UNSUPPORTED where only the
 * generic kernels apply (not bf16 / head_dim 128).
 */
SV_API int sv_decode_step_layers(sv_cache* c, int stream_id, const void* q_dev, const void* k_dev,
                                 const void* v_dev, void* o_dev, void* hip_stream);

/*
 * sv_stream_step -- one second of stream for ALL layers, sequenced natively:
 * sv_cache_evict with the three budgets, then per layer the vision chunk
 * (append, rotate Q, chunk-prefill attention), then n_text decode steps, each
 * running every layer (sv_decode_step).  This is the per-chunk loop of the
 * method (Sec. 2.1) with the projections and MLPs of the model left out: the
 * caller supplies each layer's Q/K/V up front.  Layouts (all device memory,
 * cache dtype, K un-rotated):
 *   q_vision [n_layers][n_vision][n_q_heads][head_dim]   un-rotated; MAY be rotated in place (scratch afterwards)
 *   k_vision, v_vision [n_layers][n_vision][n_kv_heads][head_dim]
 *   o_vision [n_layers][n_vision][n_q_heads][head_dim]   output
 *   q_text [n_text][n_layers][n_q_heads][head_dim], k_text / v_text
 *   [n_text][n_layers][n_kv_heads][head_dim], o_text like q_text (output)
 * n_vision == 0 skips the chunk, n_text == 0 the decoding.  decode_layers_batched
 * != 0 runs each decode step as ONE sv_decode_step_layers launch instead of
 * n_layers sv_decode_step launches (see there for when that is legitimate).
 * grid_thw as in
 * sv_cache_append (all zeros = no grid).  Errors are those of the calls it
 * sequences; on error the stream is left as the failing call left it.
 */
typedef struct sv_chunk_io {
  int32_t n_vision;
  int32_t grid_thw[3];
  void* q_vision;
  const void* k_vision;
  const void* v_vision;
  void* o_vision;
  int32_t n_text;
  const void* q_text;
  const void* k_text;
  const void* v_text;
  void* o_text;
  int32_t decode_layers_batched;
} sv_chunk_io;

SV_API int sv_stream_step(sv_cache* c, int stream_id, int64_t n_sink, int64_t vision_window,
                          int64_t text_window, const sv_chunk_io* io, int64_t* n_retained_out,
                          void* hip_stream);

/* Number of tokens currently in the stream's cache. */
SV_API int sv_cache_len(sv_cache* c, int stream_id, int64_t* n_out);

/*
 * Inspection for parity checks; SYNCHRONOUS (waits for hip_stream).  Copies
 * up to `cap` entries, in slot order: arrival ids (ids_host, [cap]) and
 * positions (pos3_host, [cap][3] as t, h, w; 1-D mode repeats the index).
 * Either pointer may be NULL.  n_out receives the cache length.  The device keeps its own count of the
 * stream's tokens (written by the eviction scan and by every registration of new tokens); this call
 * compares it with the host's bookkeeping and returns SV_ERR_STATE if the two differ.
 */
SV_API int sv_cache_retained(sv_cache* c, int stream_id, int64_t* ids_host, int32_t* pos3_host,
                      int64_t cap, int64_t* n_out, void* hip_stream);

/*
 * Inspection for parity checks; SYNCHRONOUS.  Copies the stored K (rotated) or
 * V rows of slots [slot0, slot0+n) of one layer to dst_host as
 * [n][n_kv_heads][head_dim] in the cache dtype.  which: 0 = K, 1 = V.
 */
SV_API int sv_cache_read_kv(sv_cache* c, int stream_id, int layer, int which, int64_t slot0,
                     int64_t n, void* dst_host, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SV_H_ */
