/*
 * kvmix_ref.c — CPU oracle for the KVmix hot path (arXiv 2506.08018).
 *
 * TEST INFRASTRUCTURE ONLY. Plain, slow, written from the paper; it shares no code, header,
 * table or helper with the HIP library and is only used by the tests, the smoke check and the
 * benchmark's cpu_baseline leg. Nothing in the product path may call it.
 *
 * What it computes
 *   - the group-wise asymmetric quantizer of Sec. 3.2.2 at 1, 2, 3 and 4 bits (steps 1-4 and the q_max case
 *     equation for 3-bit blocks of 11; with 1 bit the stored step is the group's range, stored as 65504 when
 *     it exceeds the fp16 range), with Keys grouped per channel and Values per token
 *     (Sec. 3.2.1), group size 32 (Sec. 4.2);
 *   - the packed-cache encoding (bit positions documented in pos_key / pos_value, the tile
 *     record in the section "tile records" below);
 *   - decode attention by its plain definition: softmax(scale * q K~^T) V~ in fp64, where
 *     K~, V~ are the dequantized packed tokens (x = q*s + min, Sec. 3.2.2 step 4) followed by
 *     the fp16 recent window (Sec. 3.3). The fused kernel of Sec. 3.4 item 2 reaches exactly
 *     this result; the fusion introduces no approximation;
 *   - the Recent Pivotal Context count num_RPC = floor(r * current_RPC) of Sec. 3.3 and the ageing it drives, with
 *     separate counts for Keys and Values (the ratios of Sec. 4.2: 20 % at 3/4 bit, 10 % at 2 bit): Keys leave
 *     the fp16 window in whole groups of 32 tokens, Values token by token.
 *
 * Readings of the paper where it is silent (each one is listed in the design document):
 *   round = round-half-to-even; scale and minimum are stored as fp16 and the quantizer uses the
 *   stored (rounded) scale; a group is 32 consecutive tokens of one channel (Keys) or 32
 *   consecutive channels of one token (Values); 3-bit blocks of 11 restart at every group
 *   (11 + 11 + 10 = 32), so in-group elements 10 and 21 are the 2-bit ones and their step is
 *   s*7/3 (the same range divided by q_max = 3); a zero-range group has scale 0 and codes 0.
 *
 * Pins (tests/test_oracle_*.py): brute-force nearest-level search, closed-form groups, the
 * round-trip bound |x - x~| <= s_i/2, bijectivity of the packing, reduction to library
 * attention when nothing is quantized, invariances of softmax attention; for the ageing: the window-count
 * sequences the formula gives for r = 0.2 and 0.1, records identical to those of the one-pass quantizer whatever
 * the order in which tokens left, attention equal to library attention over the per-token mix of sources.
 * Parity unpinned: the physical bit order, the tie rule, the fp16 storage of scale/minimum and
 * the 3-bit step reading are readings, the paper prints no worked numeric example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define D_HEAD 128
#define GROUP 32
#define TILE_TOKENS 32

enum { REF_OK = 0, REF_ERR_NULL = -1, REF_ERR_BAD_BITS = -2, REF_ERR_BAD_GROUP = -3, REF_ERR_BAD_SHAPE = -4 };

typedef struct { int32_t B, Hq, Hkv, D, group; } ref_shape;
typedef struct { int32_t k_bits, v_bits, window; } ref_layer_cfg;
typedef struct {
  uint32_t* packed;  /* tile records, see record_of() */
  uint16_t* k_win;   uint16_t* v_win;
  int32_t T_cap, W_cap, n_q, n_w, w0;
  int32_t v_lead;    /* packed Value tokens minus packed Key tokens (Sec. 3.3: the two ratios of a layer may differ) */
} ref_layer_cache; /* all pointers are host memory */
/* The sequence has n = n_q + n_w tokens. Keys of tokens [0, n_q) are packed, Values of tokens [0, n_q + v_lead);
 * every later Key / Value is an fp16 row of k_win / v_win, token t in ring slot (w0 + t - n_q) mod W_cap. */

/* ------------------------------------------------------------------ fp16 <-> binary64 */

/* IEEE binary16 bit pattern -> value (exact). */
double kvmix_ref_h2d(uint16_t h) {
  int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0) v = ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(1024 + m), e - 25);
  return sign ? -v : v;
}

/* value -> nearest binary16, ties to even, one rounding. */
uint16_t kvmix_ref_d2h(double x) {
  uint16_t sign = signbit(x) ? 0x8000u : 0;
  double a = fabs(x);
  if (isnan(a)) return sign | 0x7e00u;
  if (isinf(a)) return sign | 0x7c00u;
  if (a < ldexp(1.0, -14)) {               /* subnormal range: spacing 2^-24 */
    long q = lrint(ldexp(a, 24));          /* lrint: current mode = nearest-even */
    return sign | (uint16_t)q;             /* q == 1024 is the smallest normal, same bits */
  }
  int e;
  double m = frexp(a, &e);                 /* a = m * 2^e, m in [0.5, 1) */
  long q = lrint(ldexp(m, 11));            /* 11 significant bits: q in [1024, 2048] */
  if (q == 2048) { q = 1024; e += 1; }
  int E = e - 1 + 15;
  if (E >= 31) return sign | 0x7c00u;      /* overflow -> inf */
  return sign | (uint16_t)((E << 10) | (q - 1024));
}

static float h2f(uint16_t h) { return (float)kvmix_ref_h2d(h); }   /* exact */
static uint16_t f2h(float f) { return kvmix_ref_d2h((double)f); }  /* one rounding */

/* ------------------------------------------------------------------ quantizer (Sec. 3.2.2) */

static int qmax_of(int bits) { return (1 << bits) - 1; }

/* q_max of in-group element i: the case equation of Sec. 3.2.2 with blocks of 11 restarting
 * at each group of 32, so block positions 10 fall on i = 10 and i = 21. */
static int qmax_elem(int bits, int i) { return (bits == 3 && (i == 10 || i == 21)) ? 3 : qmax_of(bits); }

/* step of in-group element i given the stored fp16 scale: the same range over its own q_max. */
static float step_elem(int bits, int i, uint16_t scale_h) {
  float s = h2f(scale_h);
  if (qmax_elem(bits, i) == qmax_of(bits)) return s;
  return (s * 7.0f) / 3.0f;
}

/* One group of 32 fp16 values -> 32 codes + fp16 scale + fp16 zero-point (the minimum). */
void kvmix_ref_quantize_group(const uint16_t* x, int bits, uint8_t* code, uint16_t* scale_h, uint16_t* zero_h) {
  float mn = h2f(x[0]), mx = h2f(x[0]);
  for (int i = 1; i < GROUP; i++) {
    float v = h2f(x[i]);
    if (v < mn) mn = v;
    if (v > mx) mx = v;
  }
  if (mn == 0.0f) mn = 0.0f * 0.0f;                 /* -0 -> +0 */
  float range = mx - mn;                            /* step 1: s = (max - min) / q_max */
  if (range == 0.0f) range = 0.0f * 0.0f;           /* a zero-range group stores scale +0 whatever the signs of its zeros */
  float s32 = range / (float)qmax_of(bits);
  *scale_h = f2h(s32);
  if (*scale_h == 0x7C00) *scale_h = 0x7BFF;        /* a step beyond the fp16 range (1 bit only: the step is the range itself) is stored as the largest fp16 number */
  *zero_h = f2h(mn);                                /* exact: mn is an fp16 value */
  float s = h2f(*scale_h);
  for (int i = 0; i < GROUP; i++) {
    if (s == 0.0f) { code[i] = 0; continue; }
    float si = step_elem(bits, i, *scale_h);
    float t = (h2f(x[i]) - mn) / si;                /* step 2: q = round((x - min) / s) */
    float r = rintf(t);
    float hi = (float)qmax_elem(bits, i);           /* step 3: clip to [0, q_max] */
    if (r < 0.0f) r = 0.0f;
    if (r > hi) r = hi;
    code[i] = (uint8_t)r;
  }
}

/* step 4: x = q * s + min, in exact (binary64) arithmetic on the stored quantities. */
double kvmix_ref_dequant_elem(int code, int i, int bits, uint16_t scale_h, uint16_t zero_h) {
  return (double)code * (double)step_elem(bits, i, scale_h) + kvmix_ref_h2d(zero_h);
}

/* ------------------------------------------------------------------ the 3-bit word as the paper words it
 * Sec. 3.2.2: the 32 codes of a 3-bit group as blocks of 11, each block in one 32-bit integer: the block's first
 * ten elements as 3-bit fields (element j at bits [3j, 3j+3)) and its 11th element as a 2-bit field at bits
 * [30, 32). A group of 32 is 11 + 11 + 10 elements, so three words, the third with bits 30-31 unused.
 * The tile records below store the same 3 x 32 bits per group in another order (a 2-bit plane and a 1-bit
 * plane); this form exists to tie that order to the paper's sentence (tests compare the two). */
void kvmix_ref_pack_literal3(const uint8_t* code, uint32_t* words) {
  for (int w = 0; w < 3; w++) {
    words[w] = 0;
    for (int j = 0; j < 11; j++) {
      int i = 11 * w + j;
      if (i >= GROUP) break;
      if (j < 10) words[w] |= (uint32_t)(code[i] & 7u) << (3 * j);
      else words[w] |= (uint32_t)(code[i] & 3u) << 30;
    }
  }
}

void kvmix_ref_unpack_literal3(const uint32_t* words, uint8_t* code) {
  for (int i = 0; i < GROUP; i++) {
    int w = i / 11, j = i % 11;
    code[i] = (uint8_t)(j < 10 ? (words[w] >> (3 * j)) & 7u : (words[w] >> 30) & 3u);
  }
}

/* ------------------------------------------------------------------ packed tile encoding */

typedef struct { int word, bit, hword, hbit; } code_pos; /* hword < 0: no high plane */

static int words_per_tile(int bits) { return 128 * bits; } /* 32 x 128 codes, 32 bits per word */

/* Bit fields of one code given the 16-byte column l (0..63) of its 1 KiB block, the word j
 * (0..3) inside the column, the 16-bit half hh of the word and its slot (0..7) inside the half.
 *   1 bit: word 2l + j/2, bit 16hh + 8 (j%2) + 2 (slot%4) + slot/4  (32 codes per word, Sec. 3.2.2 step 4)
 *   2 bit: word 4l + j, bits [16hh + 2 slot, +2)
 *   4 bit: word 256 (slot/4) + 4l + j, bits [16hh + 4 (slot%4), +4)
 *   3 bit: code = lo + 4 hi; lo stored like a 2-bit tile, hi in a 1-bit plane after it:
 *          word 256 + 2l + j/2, bit 16hh + 8 (j%2) + 2 (slot%4) + slot/4 */
static code_pos pos_from_slots(int bits, int l, int j, int hh, int slot) {
  code_pos p; p.hword = -1; p.hbit = 0;
  if (bits == 1) { p.word = 2 * l + j / 2; p.bit = 16 * hh + 8 * (j % 2) + 2 * (slot % 4) + slot / 4; return p; }
  if (bits == 4) { p.word = 256 * (slot / 4) + 4 * l + j; p.bit = 16 * hh + 4 * (slot % 4); return p; }
  p.word = 4 * l + j; p.bit = 16 * hh + 2 * slot;
  if (bits == 3) { p.hword = 256 + 2 * l + j / 2; p.hbit = 16 * hh + 8 * (j % 2) + 2 * (slot % 4) + slot / 4; }
  return p;
}

/* Key code of token tau (0..31) and channel d (0..127) inside its tile: a word pairs two
 * adjacent channels in its halves, its slots run over channel blocks of 32 and token halves. */
static code_pos pos_key(int bits, int tau, int d) {
  int ks = d / 32, kq = (d % 32) / 8, j = (d % 8) / 2, hh = d % 2;
  int m = (tau % 8) / 4, i = 4 * (tau / 8) + tau % 4;
  return pos_from_slots(bits, 16 * kq + i, j, hh, ks + 4 * m);
}

/* Value code of token tau and channel d inside its tile: a word pairs two adjacent tokens in
 * its halves, its slots run over channel blocks of 16. */
static code_pos pos_value(int bits, int tau, int d) {
  int kq = tau / 8, j = (tau % 8) / 2, hh = tau % 2;
  int m = d / 16, i = d % 16;
  return pos_from_slots(bits, 16 * kq + i, j, hh, m);
}

static void put_code(uint32_t* tile, int bits, code_pos p, int code) {
  if (bits == 3) {
    tile[p.word] |= (uint32_t)(code & 3) << p.bit;
    tile[p.hword] |= (uint32_t)(code >> 2) << p.hbit;
  } else {
    tile[p.word] |= (uint32_t)code << p.bit;
  }
}

/* overwrite instead of OR: for a token whose neighbours in the same words are already in place */
static void set_code(uint32_t* tile, int bits, code_pos p, int code) {
  if (bits == 3) {
    tile[p.word] &= ~(3u << p.bit);
    tile[p.hword] &= ~(1u << p.hbit);
  } else {
    tile[p.word] &= ~((uint32_t)qmax_of(bits) << p.bit);
  }
  put_code(tile, bits, p, code);
}

static int get_code(const uint32_t* tile, int bits, code_pos p) {
  if (bits == 3) return (int)((tile[p.word] >> p.bit) & 3u) + 4 * (int)((tile[p.hword] >> p.hbit) & 1u);
  return (int)((tile[p.word] >> p.bit) & (uint32_t)qmax_of(bits));
}

/* codes[tau*128 + d] -> tile words (which = 0 Key, 1 Value); and back. */
void kvmix_ref_pack_tile(int which, int bits, const uint8_t* codes, uint32_t* tile) {
  memset(tile, 0, sizeof(uint32_t) * (size_t)words_per_tile(bits));
  for (int tau = 0; tau < TILE_TOKENS; tau++)
    for (int d = 0; d < D_HEAD; d++)
      put_code(tile, bits, which ? pos_value(bits, tau, d) : pos_key(bits, tau, d), codes[tau * D_HEAD + d]);
}

void kvmix_ref_unpack_tile(int which, int bits, const uint32_t* tile, uint8_t* codes) {
  for (int tau = 0; tau < TILE_TOKENS; tau++)
    for (int d = 0; d < D_HEAD; d++)
      codes[tau * D_HEAD + d] = (uint8_t)get_code(tile, bits, which ? pos_value(bits, tau, d) : pos_key(bits, tau, d));
}

/* ------------------------------------------------------------------ tile records
 * All data of one tile is one contiguous record of 32-bit words:
 *   [0, 256)                      metadata
 *   [256, 256 + 128 kb)           Key codes (tile words as above)
 *   [256 + 128 kb, + 128 vb)      Value codes
 * Metadata word 4 l + f (l = 0..63) carries two fp16 patterns, "first" in its low 16 bits:
 *   f = 0 / 1: scale / minimum of the Key groups of channels 2l (first) and 2l + 1 (second)
 *   f = 2 / 3: scale / minimum of the Value groups (token 2 (l%16), block l/16) (first) and
 *              (token 2 (l%16) + 1, block l/16) (second)                                         */
#define META_WORDS 256

int kvmix_ref_record_words(int kb, int vb) { return META_WORDS + words_per_tile(kb) + words_per_tile(vb); }

static uint32_t* record_of(const ref_layer_cache* c, int kb, int vb, int u, int tile) {
  size_t r = (size_t)u * (size_t)(c->T_cap / TILE_TOKENS) + (size_t)tile;
  return c->packed + r * (size_t)kvmix_ref_record_words(kb, vb);
}
static uint32_t* key_codes_of(uint32_t* rec) { return rec + META_WORDS; }
static uint32_t* value_codes_of(uint32_t* rec, int kb) { return rec + META_WORDS + words_per_tile(kb); }

static void meta_store(uint32_t* rec, int word, int second, uint16_t v) {
  uint32_t keep = second ? 0x0000FFFFu : 0xFFFF0000u;
  rec[word] = (rec[word] & keep) | ((uint32_t)v << (second ? 16 : 0));
}
static uint16_t meta_fetch(const uint32_t* rec, int word, int second) {
  return (uint16_t)(rec[word] >> (second ? 16 : 0));
}
/* f = 0 scale, 1 minimum */
static void key_meta_store(uint32_t* rec, int d, int f, uint16_t v) { meta_store(rec, 4 * (d / 2) + f, d % 2, v); }
static uint16_t key_meta_fetch(const uint32_t* rec, int d, int f) { return meta_fetch(rec, 4 * (d / 2) + f, d % 2); }
static void value_meta_store(uint32_t* rec, int tau, int g, int f, uint16_t v) { meta_store(rec, 4 * (16 * g + tau / 2) + 2 + f, tau % 2, v); }
static uint16_t value_meta_fetch(const uint32_t* rec, int tau, int g, int f) { return meta_fetch(rec, 4 * (16 * g + tau / 2) + 2 + f, tau % 2); }

/* ------------------------------------------------------------------ cache-level calls */

static int check_common(const ref_shape* sh, const ref_layer_cfg* cfg) {
  if (!sh || !cfg) return REF_ERR_NULL;
  if (sh->group != GROUP) return REF_ERR_BAD_GROUP;
  if (sh->D != D_HEAD || sh->B < 1 || sh->Hkv < 1 || sh->Hq < 1 || sh->Hq % sh->Hkv) return REF_ERR_BAD_SHAPE;
  int kb = cfg->k_bits, vb = cfg->v_bits;
  if (kb == 16 || vb == 16) return (kb == 16 && vb == 16) ? REF_OK : REF_ERR_BAD_BITS;
  if (kb < 1 || kb > 4 || vb < 1 || vb > 4) return REF_ERR_BAD_BITS;
  return REF_OK;
}

/* Number of OpenMP threads of the following calls (timing only; n < 1 is ignored). */
void kvmix_ref_set_num_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int kvmix_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Quantize-and-pack n_tokens tokens at token offset t0 of the packed cache.
 * Element (b, j, t, d) of k/v is at b*batch_stride + j*head_stride + t*token_stride + d*chan_stride. */
static int quantize_pack_strided(const ref_shape* sh, const ref_layer_cfg* cfg, const uint16_t* k, const uint16_t* v,
                                 int64_t k_tok, int64_t k_chan, int64_t k_unit_b, int64_t k_unit_h,
                                 int64_t v_tok, int64_t v_chan, int64_t v_unit_b, int64_t v_unit_h,
                                 int n_tokens, int t0, const ref_layer_cache* c) {
  int units = sh->B * sh->Hkv;
  int kb = cfg->k_bits, vb = cfg->v_bits;
#pragma omp parallel for schedule(static)
  for (int u = 0; u < units; u++) {
    int b = u / sh->Hkv, j = u % sh->Hkv;
    const uint16_t* ku = k + b * k_unit_b + j * k_unit_h;
    const uint16_t* vu = v + b * v_unit_b + j * v_unit_h;
    for (int tt = 0; tt < n_tokens / TILE_TOKENS; tt++) {
      uint32_t* rec = record_of(c, kb, vb, u, t0 / TILE_TOKENS + tt);
      uint8_t codes[TILE_TOKENS * D_HEAD];
      uint16_t x[GROUP]; uint8_t gc[GROUP]; uint16_t s_h, z_h;
      /* Keys: one group per channel, along the 32 tokens of the tile (Sec. 3.2.1) */
      for (int d = 0; d < D_HEAD; d++) {
        for (int tau = 0; tau < TILE_TOKENS; tau++) x[tau] = ku[(int64_t)(tt * TILE_TOKENS + tau) * k_tok + d * k_chan];
        kvmix_ref_quantize_group(x, kb, gc, &s_h, &z_h);
        key_meta_store(rec, d, 0, s_h);
        key_meta_store(rec, d, 1, z_h);
        for (int tau = 0; tau < TILE_TOKENS; tau++) codes[tau * D_HEAD + d] = gc[tau];
      }
      kvmix_ref_pack_tile(0, kb, codes, key_codes_of(rec));
      /* Values: one group per (token, 32-channel block) */
      for (int tau = 0; tau < TILE_TOKENS; tau++)
        for (int g = 0; g < D_HEAD / GROUP; g++) {
          for (int e = 0; e < GROUP; e++) x[e] = vu[(int64_t)(tt * TILE_TOKENS + tau) * v_tok + (g * GROUP + e) * v_chan];
          kvmix_ref_quantize_group(x, vb, gc, &s_h, &z_h);
          value_meta_store(rec, tau, g, 0, s_h);
          value_meta_store(rec, tau, g, 1, z_h);
          for (int e = 0; e < GROUP; e++) codes[tau * D_HEAD + g * GROUP + e] = gc[e];
        }
      kvmix_ref_pack_tile(1, vb, codes, value_codes_of(rec, kb));
    }
  }
  return REF_OK;
}

int kvmix_ref_quantize_pack(const ref_shape* sh, const ref_layer_cfg* cfg, const uint16_t* k, const uint16_t* v,
                            int64_t token_stride, int64_t head_stride, int64_t batch_stride,
                            int n_tokens, int t0, const ref_layer_cache* c) {
  int st = check_common(sh, cfg);
  if (st) return st;
  if (!k || !v || !c) return REF_ERR_NULL;
  if (cfg->k_bits == 16) return REF_ERR_BAD_BITS;
  if (n_tokens < 0 || n_tokens % TILE_TOKENS || t0 < 0 || t0 % TILE_TOKENS || t0 + n_tokens > c->T_cap) return REF_ERR_BAD_SHAPE;
  return quantize_pack_strided(sh, cfg, k, v, token_stride, 1, batch_stride, head_stride,
                               token_stride, 1, batch_stride, head_stride, n_tokens, t0, c);
}

/* ring slot of token t (both windows) */
static int slot_of(const ref_layer_cache* c, int t) {
  int W = c->W_cap, s = (c->w0 + t - c->n_q) % W;
  return s < 0 ? s + W : s;
}
/* tokens that live in the ring: from the older of the two packed fronts to the newest */
static int ring_tokens(const ref_layer_cache* c) { return c->n_w + (c->v_lead < 0 ? -c->v_lead : 0); }

/* Append one token per unit to the window ring; flush the oldest 32 into the packed cache when
 * the window holds window + 32 tokens (Sec. 3.3: older tokens are quantized, recent ones stay).
 * window == -1: nothing is flushed here, ageing is left to kvmix_ref_flush. */
int kvmix_ref_append(const ref_shape* sh, const ref_layer_cfg* cfg, const uint16_t* k_new, const uint16_t* v_new,
                     ref_layer_cache* c) {
  int st = check_common(sh, cfg);
  if (st) return st;
  if (!k_new || !v_new || !c) return REF_ERR_NULL;
  if (ring_tokens(c) >= c->W_cap) return REF_ERR_BAD_SHAPE;
  if (cfg->window >= 0 && c->v_lead != 0) return REF_ERR_BAD_SHAPE;
  int units = sh->B * sh->Hkv, W = c->W_cap;
  int slot = (c->w0 + c->n_w) % W;
  for (int u = 0; u < units; u++)
    for (int d = 0; d < D_HEAD; d++) {
      c->k_win[((size_t)u * W + slot) * D_HEAD + d] = k_new[(size_t)u * D_HEAD + d];
      c->v_win[((size_t)u * W + slot) * D_HEAD + d] = v_new[(size_t)u * D_HEAD + d];
    }
  c->n_w += 1;
  if (cfg->k_bits != 16 && cfg->window >= 0 && c->n_w == cfg->window + TILE_TOKENS) {
    if (c->n_q + TILE_TOKENS > c->T_cap) return REF_ERR_BAD_SHAPE;
    /* the oldest 32 tokens are slots w0 .. w0+31 (w0 and W_cap are multiples of 32) */
    st = quantize_pack_strided(sh, cfg, c->k_win + (size_t)c->w0 * D_HEAD, c->v_win + (size_t)c->w0 * D_HEAD,
                               D_HEAD, 1, (int64_t)sh->Hkv * W * D_HEAD, (int64_t)W * D_HEAD,
                               D_HEAD, 1, (int64_t)sh->Hkv * W * D_HEAD, (int64_t)W * D_HEAD,
                               TILE_TOKENS, c->n_q, c);
    if (st) return st;
    c->n_q += TILE_TOKENS;
    c->n_w -= TILE_TOKENS;
    c->w0 = (c->w0 + TILE_TOKENS) % W;
  }
  return REF_OK;
}

/* Dequantized packed token t of one unit as binary64: out[d] (which = 0 Key, 1 Value). */
static void dequant_token(const ref_layer_cfg* cfg, int which, const ref_layer_cache* c, int u, int t, double* out) {
  int kb = cfg->k_bits, vb = cfg->v_bits, bits = which ? vb : kb;
  int tau = t % TILE_TOKENS;
  uint32_t* rec = record_of(c, kb, vb, u, t / TILE_TOKENS);
  const uint32_t* words = which ? value_codes_of(rec, kb) : key_codes_of(rec);
  for (int d = 0; d < D_HEAD; d++) {
    uint16_t s_h, z_h; int i;
    if (which == 0) { s_h = key_meta_fetch(rec, d, 0); z_h = key_meta_fetch(rec, d, 1); i = tau; }   /* group along tokens */
    else { s_h = value_meta_fetch(rec, tau, d / GROUP, 0); z_h = value_meta_fetch(rec, tau, d / GROUP, 1); i = d % GROUP; } /* along channels */
    int code = get_code(words, bits, which ? pos_value(bits, tau, d) : pos_key(bits, tau, d));
    out[d] = kvmix_ref_dequant_elem(code, i, bits, s_h, z_h);
  }
}

/* out: [units][count][128] with count = n_q (Keys) or n_q + v_lead (Values). */
int kvmix_ref_dequant(const ref_shape* sh, const ref_layer_cfg* cfg, const ref_layer_cache* c, int which, double* out) {
  int st = check_common(sh, cfg);
  if (st) return st;
  if (!c || !out) return REF_ERR_NULL;
  if (cfg->k_bits == 16) return c->n_q == 0 ? REF_OK : REF_ERR_BAD_BITS;
  int units = sh->B * sh->Hkv, count = c->n_q + (which ? c->v_lead : 0);
  for (int u = 0; u < units; u++)
    for (int t = 0; t < count; t++)
      dequant_token(cfg, which, c, u, t, out + ((size_t)u * count + t) * D_HEAD);
  return REF_OK;
}

/* Sec. 3.3: num_RPC = floor(r * current_RPC), the product taken in binary64. */
int kvmix_ref_rpc_next(double r, int current) { return (int)floor(r * (double)current); }

/* Sec. 3.3, Fig. 4: the tokens that are no longer among the keep_k (Keys) / keep_v (Values) most recent ones are
 * quantized and join the packed part; the kept ones stay fp16. Keys can only leave in whole groups of 32 tokens
 * (Sec. 3.2.1: a Key group runs along the tokens), so the Key front moves to the largest multiple of 32 that
 * leaves at least keep_k tokens; a Value group is one token's 32 channels, so Values leave token by token.
 * Neither front moves back. */
int kvmix_ref_flush(const ref_shape* sh, const ref_layer_cfg* cfg, ref_layer_cache* c, int keep_k, int keep_v) {
  int st = check_common(sh, cfg);
  if (st) return st;
  if (!c) return REF_ERR_NULL;
  if (cfg->k_bits == 16) return REF_ERR_BAD_BITS;
  if (keep_k < 0 || keep_v < 0) return REF_ERR_BAD_SHAPE;
  int n = c->n_q + c->n_w, n_qv = c->n_q + c->v_lead;
  int nk = n - keep_k, nv = n - keep_v;
  if (nk < 0) nk = 0;
  nk -= nk % TILE_TOKENS;
  if (nk < c->n_q) nk = c->n_q;
  if (nv < n_qv) nv = n_qv;
  if (nk > c->T_cap || nv > c->T_cap) return REF_ERR_BAD_SHAPE;
  int units = sh->B * sh->Hkv, kb = cfg->k_bits, vb = cfg->v_bits, W = c->W_cap;
  for (int u = 0; u < units; u++) {
    uint16_t x[GROUP]; uint8_t gc[GROUP]; uint16_t s_h, z_h;
    for (int t0 = c->n_q; t0 < nk; t0 += TILE_TOKENS) {          /* Key tiles */
      uint32_t* rec = record_of(c, kb, vb, u, t0 / TILE_TOKENS);
      uint8_t codes[TILE_TOKENS * D_HEAD];
      for (int d = 0; d < D_HEAD; d++) {
        for (int tau = 0; tau < TILE_TOKENS; tau++) x[tau] = c->k_win[((size_t)u * W + slot_of(c, t0 + tau)) * D_HEAD + d];
        kvmix_ref_quantize_group(x, kb, gc, &s_h, &z_h);
        key_meta_store(rec, d, 0, s_h);
        key_meta_store(rec, d, 1, z_h);
        for (int tau = 0; tau < TILE_TOKENS; tau++) codes[tau * D_HEAD + d] = gc[tau];
      }
      kvmix_ref_pack_tile(0, kb, codes, key_codes_of(rec));
    }
    for (int t = n_qv; t < nv; t++) {                            /* Value tokens */
      uint32_t* rec = record_of(c, kb, vb, u, t / TILE_TOKENS);
      int tau = t % TILE_TOKENS;
      for (int g = 0; g < D_HEAD / GROUP; g++) {
        for (int e = 0; e < GROUP; e++) x[e] = c->v_win[((size_t)u * W + slot_of(c, t)) * D_HEAD + g * GROUP + e];
        kvmix_ref_quantize_group(x, vb, gc, &s_h, &z_h);
        value_meta_store(rec, tau, g, 0, s_h);
        value_meta_store(rec, tau, g, 1, z_h);
        for (int e = 0; e < GROUP; e++) set_code(value_codes_of(rec, kb), vb, pos_value(vb, tau, g * GROUP + e), gc[e]);
      }
    }
  }
  c->w0 = slot_of(c, nk);
  c->n_q = nk;
  c->n_w = n - nk;
  c->v_lead = nv - nk;
  return REF_OK;
}

/* Decode attention by definition. q, out: fp16 [B][Hq][128]. */
int kvmix_ref_decode_attn(const ref_shape* sh, const ref_layer_cfg* cfg, const uint16_t* q, const ref_layer_cache* c,
                          float softmax_scale, uint16_t* out) {
  int st = check_common(sh, cfg);
  if (st) return st;
  if (!q || !c || !out) return REF_ERR_NULL;
  if (cfg->k_bits == 16 && c->n_q != 0) return REF_ERR_BAD_BITS;
  if (c->n_q + c->n_w < 1 || c->n_q % TILE_TOKENS || ring_tokens(c) > c->W_cap) return REF_ERR_BAD_SHAPE;
  if (c->n_q + c->v_lead < 0 || c->v_lead > c->n_w) return REF_ERR_BAD_SHAPE;
  int units = sh->B * sh->Hkv, G = sh->Hq / sh->Hkv, T = c->n_q + c->n_w, W = c->W_cap, n_qv = c->n_q + c->v_lead;
  double scale = softmax_scale > 0.0f ? (double)softmax_scale : 1.0 / sqrt((double)D_HEAD);
#pragma omp parallel for schedule(dynamic, 1)
  for (int u = 0; u < units; u++) {
    int b = u / sh->Hkv, j = u % sh->Hkv;
    double* Kt = (double*)malloc(sizeof(double) * (size_t)T * D_HEAD);
    double* Vt = (double*)malloc(sizeof(double) * (size_t)T * D_HEAD);
    double* a = (double*)malloc(sizeof(double) * (size_t)T);
    for (int t = 0; t < T; t++) {                        /* packed tokens dequantized, window tokens as they are */
      int slot = slot_of(c, t);
      if (t < c->n_q) dequant_token(cfg, 0, c, u, t, Kt + (size_t)t * D_HEAD);
      else for (int d = 0; d < D_HEAD; d++) Kt[(size_t)t * D_HEAD + d] = kvmix_ref_h2d(c->k_win[((size_t)u * W + slot) * D_HEAD + d]);
      if (t < n_qv) dequant_token(cfg, 1, c, u, t, Vt + (size_t)t * D_HEAD);
      else for (int d = 0; d < D_HEAD; d++) Vt[(size_t)t * D_HEAD + d] = kvmix_ref_h2d(c->v_win[((size_t)u * W + slot) * D_HEAD + d]);
    }
    for (int hg = 0; hg < G; hg++) {
      int h = j * G + hg;                                /* query head h reads kv head h / G */
      const uint16_t* qh = q + ((size_t)b * sh->Hq + h) * D_HEAD;
      double m = -INFINITY;
      for (int t = 0; t < T; t++) {
        double acc = 0.0;
        for (int d = 0; d < D_HEAD; d++) acc += kvmix_ref_h2d(qh[d]) * Kt[(size_t)t * D_HEAD + d];
        a[t] = scale * acc;
        if (a[t] > m) m = a[t];
      }
      double l = 0.0;
      for (int t = 0; t < T; t++) { a[t] = exp(a[t] - m); l += a[t]; }
      for (int d = 0; d < D_HEAD; d++) {
        double o = 0.0;
        for (int t = 0; t < T; t++) o += a[t] * Vt[(size_t)t * D_HEAD + d];
        out[((size_t)b * sh->Hq + h) * D_HEAD + d] = kvmix_ref_d2h(o / l);
      }
    }
    free(Kt); free(Vt); free(a);
  }
  return REF_OK;
}
