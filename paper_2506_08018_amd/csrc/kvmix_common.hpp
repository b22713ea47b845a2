// Shared definitions of the KVmix HIP library (gfx950). Not used by the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/kvmix.h"

namespace kvmix {

constexpr int kD = 128;        // head dimension
constexpr int kTile = 32;      // tokens per tile = Key group length = Value group width
constexpr int kWave = 64;

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__host__ __device__ constexpr int tile_words(int bits) { return 128 * bits; }  // 32 x 128 codes
// A tile record: 256 metadata words, then the Key code section, then the Value code section.
constexpr int kMetaWords = 256;
__host__ __device__ constexpr int record_words(int k_bits, int v_bits) { return kMetaWords + tile_words(k_bits) + tile_words(v_bits); }
// 16-bit index, inside a record, of the metadata halves (f = 0 scale, 1 minimum)
__host__ __device__ constexpr int key_meta_half(int d, int f) { return 2 * (4 * (d >> 1) + f) + (d & 1); }
__host__ __device__ constexpr int value_meta_half(int tau, int g, int f) { return 2 * (4 * (16 * g + (tau >> 1)) + 2 + f) + (tau & 1); }

// Position of a code inside its tile (layout statement: include/kvmix.h).
// (l, j, hh, slot): 16-byte column, word in column, 16-bit half, slot in half.
struct CodePos { int word, bit, hword, hbit; };

__host__ __device__ inline CodePos pos_from_slots(int bits, int l, int j, int hh, int slot) {
  CodePos p;
  p.hword = -1; p.hbit = 0;
  if (bits == 1) {
    p.word = 2 * l + (j >> 1);
    p.bit = 16 * hh + 8 * (j & 1) + 2 * (slot & 3) + (slot >> 2);
    return p;
  }
  if (bits == 4) {
    p.word = 256 * (slot >> 2) + 4 * l + j;
    p.bit = 16 * hh + 4 * (slot & 3);
    return p;
  }
  p.word = 4 * l + j;
  p.bit = 16 * hh + 2 * slot;
  if (bits == 3) {
    p.hword = 256 + 2 * l + (j >> 1);
    p.hbit = 16 * hh + 8 * (j & 1) + 2 * (slot & 3) + (slot >> 2);
  }
  return p;
}

// Token / channel held by (column l, word j, half hh, slot) of a Key or Value tile.
__host__ __device__ inline void key_td(int l, int j, int hh, int slot, int& tau, int& d) {
  const int i = l & 15, kq = l >> 4, ks = slot & 3, m = slot >> 2;
  d = 32 * ks + 8 * kq + 2 * j + hh;
  tau = 8 * (i >> 2) + 4 * m + (i & 3);
}
__host__ __device__ inline void value_td(int l, int j, int hh, int slot, int& tau, int& d) {
  const int i = l & 15, kq = l >> 4;
  d = 16 * slot + i;
  tau = 8 * kq + 2 * j + hh;
}

// x = code * s_i + min (Sec. 3.2.2 step 4) of token tau, channel d of a tile record, in fp32 (multiply, then add);
// which = 0 Key, 1 Value. The straightforward form, for the helper kernels that are not bound by it.
__device__ inline float dequant_elem(const uint32_t* rec, int k_bits, int v_bits, int which, int tau, int d) {
  const uint16_t* meta = reinterpret_cast<const uint16_t*>(rec);
  const int bits = which ? v_bits : k_bits;
  const uint32_t* words = rec + kMetaWords + (which ? tile_words(k_bits) : 0);
  int l, j, hh, slot, gi, ms, mz;
  if (which == 0) {
    const int ks = d / 32, kq = (d % 32) / 8, m = (tau % 8) / 4, i = 4 * (tau / 8) + tau % 4;
    l = 16 * kq + i; j = (d % 8) / 2; hh = d % 2; slot = ks + 4 * m;
    ms = key_meta_half(d, 0); mz = key_meta_half(d, 1); gi = tau;
  } else {
    l = 16 * (tau / 8) + d % 16; j = (tau % 8) / 2; hh = tau % 2; slot = d / 16;
    ms = value_meta_half(tau, d / 32, 0); mz = value_meta_half(tau, d / 32, 1); gi = d % 32;
  }
  const CodePos p = pos_from_slots(bits, l, j, hh, slot);
  int code;
  if (bits == 3) code = ((words[p.word] >> p.bit) & 3u) + 4 * ((words[p.hword] >> p.hbit) & 1u);
  else code = (words[p.word] >> p.bit) & ((1u << bits) - 1u);
  const float s = (float)__builtin_bit_cast(half_t, meta[ms]);
  const float mn = (float)__builtin_bit_cast(half_t, meta[mz]);
  const float si = (bits == 3 && (gi == 10 || gi == 21)) ? (s * 7.0f) / 3.0f : s;
  const float prod = (float)code * si;
  return prod + mn;
}

// Launch descriptors filled by the C-ABI layer (host) and passed by value.
struct QuantArgs {
  // The token sequence that is quantized: its rows [0, n_ring) are the ring slots (ring_w0 + r) % W_cap of the two
  // fp16 windows ([units][W_cap][128]), every later row r is row r - n_ring of the input. Tile t takes rows
  // 32 t .. 32 t + 31.
  const uint16_t* k; const uint16_t* v;
  int64_t k_tok, k_unit_b, k_unit_h;            // Key input: channel stride 1
  int64_t v_tok, v_unit_b, v_unit_h;            // Value input: channel stride 1
  const uint16_t* k_ring; const uint16_t* v_ring;
  int n_ring, ring_w0, W_cap;
  uint32_t* packed;
  int tiles_cap;   // tiles per unit in the packed cache
  int tile0;       // first destination tile
  int Hkv;
  // Ageing with separate fronts (every row comes from the ring, row r of the launch is token 32*tile0 + r): the Key
  // side is written for the destination tiles [k_tile_a, k_tile_b) only, the Value side for the tokens
  // [v_tok_a, v_tok_b) only; everything else in the records is left as it is.
  int k_tile_a, k_tile_b, v_tok_a, v_tok_b;
};

struct DequantArgs {
  const uint32_t* packed;
  float* out; int tiles_cap; int n_tokens; int k_bits; int v_bits; int which;   // out: [units][n_tokens][128]
};

struct AppendArgs {
  const uint16_t* k_new; const uint16_t* v_new;   // element (b, j, i, d) at b*batch + j*head + i*tok + d
  int64_t tok, head, batch;
  uint16_t* k_win; uint16_t* v_win;
  int W_cap; int slot; int n; int units; int Hkv;   // tokens i = 0..n-1 go to ring slots (slot + i) % W_cap
};

struct AttnArgs {
  const uint16_t* q; uint16_t* out;
  const uint32_t* packed;
  const uint16_t* k_win; const uint16_t* v_win;
  // fused append: the newest token of every unit ([units][128] each) is not in the window arrays yet but counted
  // in n_w; the wave that takes the window tile of ring slot new_slot reads it from here and stores it
  const uint16_t* k_new; const uint16_t* v_new;
  uint16_t* k_win_w; uint16_t* v_win_w;
  int new_slot;           // -1: nothing to append
  float* part;            // partials: [units][n_parts][G][kD + 2], the first n_splits of a unit written by this launch
  int n_parts;            // n_splits, plus one when an earlier launch left the partial of the tokens between two fronts
  uint32_t* counters;     // [units] arrival counters (zero before and after every call)
  int tiles_cap, W_cap, n_tiles, n_w, w0;
  int Hq, Hkv, n_splits;
  int items_q, items_r;   // (window tiles + packed tiles) divided by n_splits: quotient and remainder
  float scale_log2;       // softmax_scale * log2(e)
};

// Tokens [t_begin, t_end) of every unit, each Key and each Value from where it lives (packed before its front, the
// fp16 ring from it on): one partial (reference, sum of numerators, unnormalized output) per (unit, head) into
// slot part_index of the partials array.
struct MixedArgs {
  const uint16_t* q; const uint32_t* packed; const uint16_t* k_win; const uint16_t* v_win;
  float* part; int n_parts, part_index;
  int tiles_cap, W_cap, k_bits, v_bits;
  int n_qk, n_qv;          // the two fronts
  int t_begin, t_end;      // t_begin is a multiple of 32
  int slot_begin;          // ring slot of token t_begin
  int G, G_main;           // query heads per kv head; heads per (unit, block) pair of the main kernel's partials (min(G, 8))
  float scale_log2;
};

hipError_t launch_quantize_pack(const QuantArgs& a, int k_bits, int v_bits,
                                int n_tiles, int units, hipStream_t s);
hipError_t launch_quantize_fronts(const QuantArgs& a, int k_bits, int v_bits,
                                  int n_tiles, int units, hipStream_t s);
hipError_t launch_mixed_fronts(const MixedArgs& a, int units, hipStream_t s);
hipError_t launch_dequant(const DequantArgs& a, int units, hipStream_t s);
hipError_t launch_append(const AppendArgs& a, hipStream_t s);
hipError_t launch_stream_read(const void* buf, size_t bytes, int workgroups, int threads, uint32_t* sink, hipStream_t s);
hipError_t launch_decode_attn(const AttnArgs& a, int k_bits, int v_bits, int G, int units, hipStream_t s);

}  // namespace kvmix
