/*
 * kvmix.h — C-ABI boundary of the KVmix hot path on MI355X (gfx950).
 *
 * The library implements the two data-parallel parts of KVmix (arXiv 2506.08018):
 *   part 1  group-wise asymmetric min/max quantization of the KV cache at a layer's own
 *           Key / Value bit-width, with bit-packing into 32-bit words (paper Sec. 3.2.1,
 *           3.2.2 incl. the unnumbered q_max equation for the 3-bit block of ten 3-bit and one
 *           2-bit element), applied to tokens that leave the full-precision recent window
 *           (Recent Pivotal Context, Sec. 3.3, Fig. 4); and
 *   part 2  decode attention that dequantizes the packed codes inside the dot products and never
 *           materializes an fp16 copy of the packed cache (Sec. 3.4 item 2), over
 *           [packed old tokens || fp16 recent window].
 * The per-layer bit table (Sec. 3.1, Sec. 4.2) is an input.
 *
 * Conventions
 *   - plain C, every pointer is DEVICE memory unless marked "host"; structs are host memory.
 *   - fp16 values travel as uint16_t bit patterns (IEEE binary16).
 *   - every entry point returns 0 (KVMIX_OK) or a negative kvmix_status; arguments are
 *     validated on the host before anything is launched: a failing call launches nothing
 *     and writes nothing.
 *   - the caller owns every buffer; the library allocates nothing and keeps no state
 *     besides the last HIP error code. Work is enqueued on `stream` (a hipStream_t passed
 *     as void*, NULL = default stream) and the call returns without synchronizing.
 *   - one "unit" is one (batch b, kv head j) pair, u = b*Hkv + j. Query head h reads kv head
 *     h / G, G = Hq / Hkv: 1, 2, 4 or a multiple of 8 up to 512 (multi-query attention: Hkv = 1; a head count
 *     that is no such multiple is padded by the caller with zero query rows, whose outputs are ignored).
 *   - D = 128 and group = 32 are the only supported head dimension / group size
 *     (the paper's setting, Sec. 4.2).
 *
 * Packed cache layout (per layer): one buffer `packed` of [units][T_cap/32] tile records
 *   A "tile" is 32 consecutive tokens x 128 channels of one unit. Token index inside the tile
 *   tau = 0..31, channel d = 0..127.
 *   Keys are quantized per channel: a group is the 32 tokens of a tile for one channel
 *   (Sec. 3.2.1: tensor viewed as [B*nh*D, T], cut into groups of 32 along T).
 *   Values are quantized per token: a group is 32 consecutive channels of one token, g = d/32.
 *   Everything a tile needs is contiguous: its record is 256 + 128*k_bits + 128*v_bits 32-bit
 *   words = [metadata: 256 words][Key codes: 128*k_bits words][Value codes: 128*v_bits words]
 *   (3072 bytes for 2/2 bit, 5120 for 4/4). Record r = u*(T_cap/32) + tile starts at word
 *   r * record_words.
 *   Metadata. "lane" l = 0..63 names a 16-byte column; word 4*l + f holds two fp16 values, the
 *   first in bits [0,16), the second in bits [16,32):
 *     f = 0: Key scale s of channels 2l, 2l+1        f = 1: Key group minimum of the same two
 *     f = 2: Value scale of groups (tau, g) = (2*(l%16), l/16) and (2*(l%16) + 1, l/16)
 *     f = 3: Value group minimum of the same two groups
 *   Codes. Inside its code section the position of every code is given below; l = 16*kq + i.
 *     Key code (tau, d):   ks = d/32, kq = (d%32)/8, j = (d%8)/2, hh = d%2,
 *                          m = (tau%8)/4, i = 4*(tau/8) + tau%4, slot = ks + 4*m
 *     Value code (tau, d): kq = tau/8, j = (tau%8)/2, hh = tau%2, i = d%16, slot = d/16
 *     1-bit: word 2*l + j/2, bit 16*hh + 8*(j%2) + 2*(slot%4) + slot/4 (32 codes per word; the stored scale
 *            is the group's range).
 *     2-bit: word 4*l + j, bits [16*hh + 2*slot, +2).
 *     4-bit: word 256*(slot/4) + 4*l + j, bits [16*hh + 4*(slot%4), +4).
 *     3-bit: code = lo + 4*hi. The 2-bit plane `lo` is stored exactly like a 2-bit section
 *            (256 words), followed by the 1-bit plane `hi` (128 words): word 256 + 2*l + j/2,
 *            bit 16*hh + 8*(j%2) + 2*(slot%4) + slot/4.
 *            The two elements of every group that the paper stores with 2 bits (in-group
 *            index 10 and 21: the 11th element of the first and second block of 11) have
 *            hi = 0 by construction, so a group occupies 3 words = 30*3 + 2*2 + 2 unused bits,
 *            the density of the paper's 11-per-word packing.
 *   Unused bits are zero.
 *
 * Recent window (fp16, ring buffer of W_cap slots, W_cap % 32 == 0, W_cap >= window + 32)
 *   k_win, v_win : [units][W_cap][128]   (channel contiguous: appending a token writes one full row of each)
 *   The sequence has n = n_q + n_w tokens; token t >= n_q sits in slot (w0 + t - n_q) % W_cap of both windows, so
 *   the n_w window tokens are slots (w0 + r) % W_cap, r = 0..n_w-1, oldest first; w0 % 32 == 0. Slots outside the
 *   live tokens are never read (they may hold anything, NaN patterns included).
 *   Keys and Values may age at fronts of their own (Sec. 3.3: the ratio of a layer's Keys and Values may differ):
 *   Keys of tokens [0, n_q) are packed, Values of tokens [0, n_q + v_lead). A Key group runs along 32 tokens, so
 *   the Key front n_q is a multiple of 32; a Value group is one token's 32 channels, so the Value front may stand
 *   anywhere, also inside a tile (the tile's record then holds the Value codes and metadata of its first tokens
 *   only, the rest of those fields is unspecified until their tokens arrive). With v_lead < 0 the Value rows of
 *   tokens [n_q + v_lead, n_q) are still in v_win, in the slots the formula above gives (the ring then holds
 *   n_w - v_lead tokens, which must fit W_cap). v_lead == 0, Keys and Values ageing together, is what every call
 *   but kvmix_flush produces, and the only state the fixed-window calls (window >= 0) accept.
 *
 * Numeric preconditions (not checked on the device)
 *   - all K / V / q inputs are finite (Sec. 3.2.2 defines the quantizer on real numbers only);
 *   - the quantizer is total on finite inputs: with 2-4 bits the scale (max - min)/q_max of fp16 inputs is always
 *     an fp16 number; a 1-bit scale (the range itself) that exceeds 65504 is stored as 65504 (the codes are taken
 *     against that stored scale, so the upper level dequantizes to min + 65504);
 *   - attention folds q*scale products into fp16 matrix-core operands: |q[h][d]| * s[d] < 16384 for every
 *     Key group scale s[d], and softmax numerators of up to 64 times a Value group scale: s < 1024 for every
 *     Value scale; both hold for any cache whose values stay below ~10^3 in magnitude at |q| <= 8.
 */
#ifndef KVMIX_H_
#define KVMIX_H_

#include <stddef.h>
#include <stdint.h>

/* ---- Reaching codes, scales and minima inside a tile record (the layout statement above as code).
 * All indices are relative to the record's first 32-bit word (or first 16-bit half-word where said). */
static inline int kvmix_record_words(int k_bits, int v_bits) { return 256 + 128 * k_bits + 128 * v_bits; }
static inline int kvmix_key_codes_word(void) { return 256; }
static inline int kvmix_value_codes_word(int k_bits) { return 256 + 128 * k_bits; }
/* 16-bit half-word index of the fp16 scale (f = 0) / minimum (f = 1) of the Key group of channel d (0..127) */
static inline int kvmix_key_meta_half(int d, int f) { return 2 * (4 * (d / 2) + f) + d % 2; }
/* the same for the Value group of token tau (0..31), channel block g = d / 32 (0..3) */
static inline int kvmix_value_meta_half(int tau, int g, int f) { return 2 * (4 * (16 * g + tau / 2) + 2 + f) + tau % 2; }
/* Position of the code of (token tau, channel d) inside its code section: its low `bits` (2 for 3-bit codes)
 * start at bit *bit of word *word; for 3-bit codes the third bit is bit *hbit of word *hword (else *hword = -1). */
static inline void kvmix_code_position(int is_value, int bits, int tau, int d, int* word, int* bit, int* hword, int* hbit) {
  int l, j, hh, slot;
  if (!is_value) {
    const int ks = d / 32, kq = (d % 32) / 8, m = (tau % 8) / 4, i = 4 * (tau / 8) + tau % 4;
    l = 16 * kq + i; j = (d % 8) / 2; hh = d % 2; slot = ks + 4 * m;
  } else {
    l = 16 * (tau / 8) + d % 16; j = (tau % 8) / 2; hh = tau % 2; slot = d / 16;
  }
  *hword = -1; *hbit = 0;
  if (bits == 1) { *word = 2 * l + j / 2; *bit = 16 * hh + 8 * (j % 2) + 2 * (slot % 4) + slot / 4; return; }
  if (bits == 4) { *word = 256 * (slot / 4) + 4 * l + j; *bit = 16 * hh + 4 * (slot % 4); return; }
  *word = 4 * l + j; *bit = 16 * hh + 2 * slot;
  if (bits == 3) { *hword = 256 + 2 * l + j / 2; *hbit = 16 * hh + 8 * (j % 2) + 2 * (slot % 4) + slot / 4; }
}

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVMIX_OK = 0,
  KVMIX_ERR_NULL = -1,      /* a required pointer is NULL */
  KVMIX_ERR_BAD_BITS = -2,  /* bits not in {1,2,3,4}, or 16 for one of K/V only */
  KVMIX_ERR_BAD_GROUP = -3, /* group != 32 */
  KVMIX_ERR_BAD_SHAPE = -4, /* D != 128, Hq % Hkv, G not 1, 2, 4 or a multiple of 8, counts not multiples of 32, capacity exceeded */
  KVMIX_ERR_ALIGN = -5,     /* a pointer is not 16-byte aligned or a stride is not a multiple of 8 elements */
  KVMIX_ERR_WORKSPACE = -6, /* workspace too small */
  KVMIX_ERR_HIP = -7        /* a HIP call failed; see kvmix_last_hip_error() */
} kvmix_status;

/* Cache geometry of one layer (Sec. 3.2.1: cache shape [B, nh, T, D]). */
typedef struct {
  int32_t B;     /* batch */
  int32_t Hq;    /* query heads */
  int32_t Hkv;   /* key/value heads */
  int32_t D;     /* head dimension, must be 128 */
  int32_t group; /* quantization group size, must be 32 (Sec. 4.2) */
} kvmix_shape;

/* One row of the per-layer bit table (Sec. 3.1 step 3, Sec. 4.2) plus the window length. */
typedef struct {
  int32_t k_bits; /* 1, 2, 3, 4, or 16 (= keep the whole layer in the fp16 window) */
  int32_t v_bits; /* same set; 16 only together with k_bits == 16 */
  int32_t window; /* number of most recent tokens kept in fp16 (the RPC count), multiple of 32: the appending calls
                     flush 32 tokens whenever window + 32 are held. -1: the appending calls flush nothing, ageing is
                     driven by kvmix_flush (Sec. 3.3's count, kvmix_rpc_next) */
} kvmix_layer_cfg;

/* One layer's cache: caller-owned device buffers, host-side counters. */
typedef struct {
  uint32_t* packed;  /* tile records (may be NULL when k_bits == 16) */
  uint16_t* k_win;   uint16_t* v_win;
  int32_t T_cap; /* capacity of the packed part in tokens, multiple of 32 */
  int32_t W_cap; /* window slots, multiple of 32, >= window + 32 */
  int32_t n_q;   /* packed tokens (multiple of 32), the oldest n_q tokens of the sequence */
  int32_t n_w;   /* valid window tokens */
  int32_t w0;    /* ring start slot (multiple of 32) */
  int32_t v_lead; /* packed Value tokens minus packed Key tokens, 0 unless kvmix_flush moved the fronts apart */
} kvmix_layer_cache;

int kvmix_version(void);
const char* kvmix_strerror(int status);
/* HIP error code (hipError_t as int) of the most recent KVMIX_ERR_HIP on this thread's process. */
int kvmix_last_hip_error(void);

/* Byte sizes of the cache buffers for capacities (T_cap, W_cap). Any output pointer may be
 * NULL. packed_b is the size of `packed` (0 for 16 bit), win_b of EACH of k_win, v_win. */
int kvmix_cache_bytes(const kvmix_shape* shape, const kvmix_layer_cfg* cfg, int T_cap, int W_cap,
                      size_t* packed_b, size_t* win_b);

/* Workspace needed by kvmix_decode_attn for any context up to T_max packed tokens (split
 * partials + arrival counters, and the partial of the tokens between the two fronts when v_lead != 0). The
 * workspace must be zero-filled once before first use; every call leaves the counters zero again. */
int kvmix_workspace_bytes(const kvmix_shape* shape, int T_max, size_t* bytes);

/* Part 1 (Sec. 3.2.2 steps 1-4, Sec. 3.4 item 1). Quantize n_tokens (multiple of 32) fp16
 * tokens of K and V and write codes, scales and minima into the tile records at token offset t0
 * (multiple of 32, t0 + n_tokens <= T_cap). Element (b, j, t, d) of k_fp16 / v_fp16 is at
 * index b*batch_stride + j*head_stride + t*token_stride + d (strides in elements, multiples
 * of 8). Per group: mn/mx by fp16 comparison; s = fp16((mx - mn) / qmax) with fp32
 * arithmetic; code = clamp(rint((x - mn) / s_i), 0, qmax_i) in fp32 with round-half-even,
 * where for 3 bit the in-group elements 10 and 21 use qmax_i = 3 and s_i = (s*7)/3;
 * a zero scale gives all-zero codes and is stored as +0; a 1-bit scale above 65504 is stored as 65504; the stored zero-point is mn (-0 stored as +0).
 * Does not touch n_q / n_w (the caller sets cache->n_q). Inputs must be finite. */
int kvmix_quantize_pack(const kvmix_shape* shape, const kvmix_layer_cfg* cfg,
                        const uint16_t* k_fp16, const uint16_t* v_fp16,
                        int64_t token_stride, int64_t head_stride, int64_t batch_stride,
                        int n_tokens, int t0, const kvmix_layer_cache* cache, void* stream);

/* Decode-time append of one token per sequence (Sec. 3.3, Fig. 4; Sec. 3.4 item 1):
 * k_new, v_new are fp16 [B][Hkv][128]. The token goes into the next window slot; when the
 * window then holds window + 32 tokens, the oldest 32 are quantized exactly as in
 * kvmix_quantize_pack and written at token offset n_q of the packed cache (joining the new codes to the
 * historical cache is an offset write into the pre-allocated buffer). Updates n_q, n_w, w0 in *cache (host).
 * With k_bits == 16 or window == -1 nothing is ever flushed (the ring must have a free slot). */
int kvmix_append(const kvmix_shape* shape, const kvmix_layer_cfg* cfg,
                 const uint16_t* k_new, const uint16_t* v_new,
                 kvmix_layer_cache* cache, void* stream);

/* Part 2 (Sec. 3.4 item 2; Sec. 3.2.2 dequantization x = q*s + min). For every query head h:
 *   a_t  = softmax_scale * sum_d q[h][d] * Kt[t][d]           over all n_q + n_w tokens,
 *   out  = sum_t softmax(a)_t * Vt[t][:]                       (no mask: one decode query)
 * where Kt, Vt are the dequantized packed tokens followed by the fp16 window tokens.
 * q, out: fp16 [B][Hq][128]. softmax_scale <= 0 selects 1/sqrt(D). Accumulation is fp32.
 * n_splits: number of context splits per unit (split-K), 0 = chosen by the library.
 * workspace: see kvmix_workspace_bytes (may be NULL when the effective n_splits is 1 and v_lead == 0).
 * With v_lead != 0 the tokens from the tile of the older front up to the tile end of the younger one (each Key and
 * each Value taken from where it lives: packed and dequantized, or fp16) are worked on by a launch of their own that
 * goes first and leaves one more partial in the workspace, which the main launch's merge includes. */
int kvmix_decode_attn(const kvmix_shape* shape, const kvmix_layer_cfg* cfg, const uint16_t* q,
                      const kvmix_layer_cache* cache, float softmax_scale, uint16_t* out,
                      void* workspace, size_t workspace_bytes, int n_splits, void* stream);

/* kvmix_decode_attn for callers that cannot allocate or hand over a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments and result, but the split partials and
 * arrival counters live in a fixed array of KVMIX_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (each GPU the library runs on holds its own copy until the process ends). The call allocates nothing.
 * It returns KVMIX_ERR_WORKSPACE when the (explicit or library-chosen) split count needs more than the array
 * holds: units * n_splits * G * 520 bytes + 4 bytes per unit rounded up to 256. The first call on a device looks
 * up the array's address and clears its counters on `stream`; make that call with the device current and outside
 * any graph capture. All calls on one GPU share the array: calls that overlap in time on one GPU (different
 * streams) race; calls on one stream, or otherwise ordered, are safe. */
#define KVMIX_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
int kvmix_decode_attn_static(const kvmix_shape* shape, const kvmix_layer_cfg* cfg, const uint16_t* q,
                             const kvmix_layer_cache* cache, float softmax_scale, uint16_t* out,
                             int n_splits, void* stream);

/* kvmix_append for n_tokens consecutive new tokens per sequence (chunked prefill, speculative decoding): the same
 * counters, tile records and live window tokens as n_tokens calls of kvmix_append in a row, in at most two
 * launches: one quantize-and-pack launch over all tiles that fall due (their tokens are read from the ring or
 * straight from k_new / v_new: Sec. 3.4 item 1, new states are quantized and joined to the cache without a pass of
 * their own through memory), then one copy of the new tokens that stay in the window. Element (b, j, i, d)
 * of k_new / v_new is at b*batch_stride + j*head_stride + i*token_stride + d (strides in elements, multiples of 8,
 * token_stride >= 128; pointers 16-byte aligned). Capacity (T_cap, W_cap) is checked for the whole call before
 * anything is launched. Ring slots outside the n_w live tokens are unspecified afterwards. */
int kvmix_append_tokens(const kvmix_shape* shape, const kvmix_layer_cfg* cfg,
                        const uint16_t* k_new, const uint16_t* v_new,
                        int64_t token_stride, int64_t head_stride, int64_t batch_stride, int n_tokens,
                        kvmix_layer_cache* cache, void* stream);

/* One decode step of a layer: kvmix_append followed by kvmix_decode_attn, same arguments and the same result.
 * The append is done inside the attention launch: the wave that reads the window tile of the new slot takes
 * that row from k_new / v_new and stores it into the window (Sec. 3.4 item 1 in spirit: no separate pass over
 * the cache for the new token). On the step where the window overflows one quantize-and-pack launch over the 32
 * oldest window tokens goes first (with window == 0 the new token is one of them: append, pack, then a plain
 * attention launch). With window == -1 nothing is flushed; when v_lead != 0 and the new token shares its tile with
 * the younger front, the append is a launch of its own. Updates n_q, n_w, w0 in *cache (host). k_new, v_new (16-byte aligned) must stay valid until
 * the launches have run. */
int kvmix_decode_step(const kvmix_shape* shape, const kvmix_layer_cfg* cfg,
                      const uint16_t* k_new, const uint16_t* v_new, const uint16_t* q,
                      kvmix_layer_cache* cache, float softmax_scale, uint16_t* out,
                      void* workspace, size_t workspace_bytes, int n_splits, void* stream);

/* Sec. 3.3: num_RPC = floor(r * current_RPC) for a layer's Keys (r_k, current_k) and Values (r_v, current_v), the
 * products taken in binary64; current_RPC = new tokens of this step + RPCs kept so far. Host arithmetic only.
 * Ratios outside [0, 1] or negative counts: KVMIX_ERR_BAD_SHAPE. (Sec. 4.2 uses r = 0.2 at 3/4 bit, 0.1 at 2 bit.) */
int kvmix_rpc_next(double r_k, double r_v, int current_k, int current_v, int* num_k, int* num_v);

/* Ageing by count (Sec. 3.3, Fig. 4): tokens that are no longer among the keep_k most recent lose their fp16 Key,
 * those no longer among the keep_v most recent their fp16 Value; both are quantized as in kvmix_quantize_pack, from
 * the ring, in one launch. Keys leave in whole groups of 32 tokens: the Key front moves to the largest multiple of
 * 32 that is <= n - keep_k; Values leave token by token: the Value front moves to n - keep_v. Neither front moves
 * back (a count larger than what is held changes nothing). Updates n_q, n_w, w0, v_lead in *cache (host).
 * KVMIX_ERR_BAD_SHAPE when a front would pass T_cap, KVMIX_ERR_BAD_BITS for a 16-bit layer. */
int kvmix_flush(const kvmix_shape* shape, const kvmix_layer_cfg* cfg, kvmix_layer_cache* cache,
                int keep_k, int keep_v, void* stream);

/* Test helper: dequantize the packed tokens back to fp32 (x = code*s_i + mn evaluated in fp32), which = 0 for K
 * (n_q tokens), 1 for V (n_q + v_lead tokens); out is [units][that count][128]. */
int kvmix_dequant(const kvmix_shape* shape, const kvmix_layer_cfg* cfg,
                  const kvmix_layer_cache* cache, int which, float* out, void* stream);

/* Benchmark helper: a load-only pass over `bytes` bytes of device memory at `buf` (16-byte aligned) in the
 * attention kernel's launch shape: `workgroups` workgroups of `threads` threads (multiple of 64, <= 768), each
 * reading one contiguous span with 16-byte loads under the same cache policy. Nothing is computed or written
 * (`sink`, 4 bytes of device memory or NULL, is only there to keep the loads alive). Timed next to the attention
 * launch it gives the read rate a launch of that shape and size can reach on the machine at hand. */
int kvmix_stream_read(const void* buf, size_t bytes, int workgroups, int threads, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVMIX_H_ */
