// Quantize-and-pack, dequantize (test helper) and window-append kernels for gfx950.
//
// Paper Sec. 3.2.1 (Keys grouped per channel, Values per token), Sec. 3.2.2 (group-wise
// min/max quantizer, steps 1-4, 3-bit block of 11 with q_max = 3 for its 11th element),
// Sec. 3.4 item 1 (quantize and append into the historical cache in one kernel).
//
// Built with -ffp-contract=off: the code arithmetic is specified operation by operation
// (fp32 subtract, IEEE divide, round-half-even) so that codes are reproducible bit for bit.
#include "kvmix_common.hpp"

namespace kvmix {

namespace {

template <int BITS>
__device__ __forceinline__ float step_of(float s, int i) {
  if (BITS == 3 && (i == 10 || i == 21)) return (s * 7.0f) / 3.0f;  // same range over q_max = 3
  return s;
}

template <int BITS>
__device__ __forceinline__ int qmax_of(int i) {
  if (BITS == 3 && (i == 10 || i == 21)) return 3;
  return (1 << BITS) - 1;
}

// value of lane (l ^ 1) / (l ^ 2) of each quad
__device__ __forceinline__ uint32_t quad_x1(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false); }
__device__ __forceinline__ uint32_t quad_x2(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false); }

// Codes travel as "biased codes": the bit pattern of the float 1.5 * 2^23 + code, i.e. kBias + code. Adding
// 1.5 * 2^23 to a value in [0, 2^22) rounds it to an integer (ties to even) in one operation and leaves that
// integer in the low mantissa bits; the low 16 bits of kBias are zero.
constexpr float kMagic = 12582912.0f;
constexpr uint32_t kBias = 0x4B400000u;

// Scale, minimum and bracketing reciprocal steps of one group from its extremes (fp32 images of fp16 values).
struct GroupParams { float mn, s, inv_lo, inv_hi, inv2_lo, inv2_hi; bool slow; uint16_t scale_h, zero_h; };
template <int BITS>
__device__ __forceinline__ GroupParams group_params(float mn, float mx) {
  GroupParams g;
  if (mn == 0.0f) mn = 0.0f;                      // -0 -> +0
  float range = mx - mn;
  if (range == 0.0f) range = 0.0f;                // a zero-range group stores scale +0 whatever the signs of its zeros
  const float s32 = range / (float)((1 << BITS) - 1);
  // round-to-nearest-even; a 1-bit step (the range itself) beyond the fp16 range is stored as the largest fp16 number
  const half_t sh = (half_t)(BITS == 1 ? fminf(s32, 65504.0f) : s32);
  g.mn = mn;
  g.s = (float)sh;
  g.scale_h = __builtin_bit_cast(uint16_t, sh);
  g.zero_h = __builtin_bit_cast(uint16_t, (half_t)mn);
  // 1 / s_i bracketed from below and above by 2^-19 relative: far more than the errors of the hardware
  // reciprocal (1 ulp), of the products below and of the fp32 rounding of the true quotient taken together
  // (under 2^-21). 0 for a zero scale: every product, hence every code, is then 0.
  const float inv = g.s != 0.0f ? __builtin_amdgcn_rcpf(g.s) : 0.0f;
  g.inv_lo = inv * (1.0f - 0x1p-19f);
  g.inv_hi = inv * (1.0f + 0x1p-19f);
  g.inv2_lo = g.inv_lo * (3.0f / 7.0f);          // the step s * 7 / 3 of the two 2-bit elements of a 3-bit group
  g.inv2_hi = g.inv_hi * (3.0f / 7.0f);
  // Only when the stored scale is a rounded image of range / q_max to fp16's full precision is every quotient
  // at most q_max * (1 + 2^-11) and the upper clip idle. A subnormal scale (rounded with a larger relative error)
  // or a saturated 1-bit scale sends the whole group down the exact path, which clips.
  g.slow = (g.s != 0.0f && g.s < 0x1p-14f) || (BITS == 1 && g.s >= 65504.0f);
  return g;
}

// code = clamp(rint((x - mn) / s_i)) with the IEEE quotient rounded to fp32 first. The quotient q lies strictly
// between (x - mn) * inv_lo and (x - mn) * inv_hi, and so does its fp32 image; rounding to an integer is
// monotone, so when both products round to the same integer (each with the single rounding of a fused
// multiply-add onto kMagic), that integer is the code. quantize_fast reports the other cases - the quotient
// within 2^-18 relative of k + 1/2, rare - and the caller redoes a small batch of elements with
// quantize_exact when any of them was one. x >= mn always, and only the exact path needs the upper clip.
// d: x - mn in fp32; i: index of the element inside its group. Both return biased codes.
template <int BITS>
__device__ __forceinline__ uint32_t quantize_fast(float d, const GroupParams& g, int i, bool& near) {
  const bool two_bit = BITS == 3 && (i == 10 || i == 21);
  const float lo = __builtin_fmaf(d, two_bit ? g.inv2_lo : g.inv_lo, kMagic);
  const float hi = __builtin_fmaf(d, two_bit ? g.inv2_hi : g.inv_hi, kMagic);
  near |= lo != hi;
  return __builtin_bit_cast(uint32_t, lo);
}
template <int BITS>
__device__ __forceinline__ uint32_t quantize_exact(float d, const GroupParams& g, int i) {
  if (g.s == 0.0f) return kBias;
  const float r = __builtin_rintf(d / step_of<BITS>(g.s, i));
  return kBias + (uint32_t)fminf(fmaxf(r, 0.0f), (float)qmax_of<BITS>(i));
}
// x - mn in fp32 for an fp16 x: one fused operation (x * 1 - mn), rounded once like the subtraction
__device__ __forceinline__ float diff(half_t x, float mn) { return __builtin_fmaf((float)x, 1.0f, -mn); }

__device__ __forceinline__ half2_t as_half2(uint32_t w) { return __builtin_bit_cast(half2_t, w); }

// Number of 32-bit word accumulators a lane fills for one code section before the lanes of its quad are
// combined: words i = 0..15 of its (kq, j) column group; 4-bit sections have two chunks. 1-bit sections
// consist of the bit plane alone (the `hi` words below, stored at the start of the section).
template <int BITS> constexpr int acc_words() { return BITS == 4 ? 32 : 16; }

// Final step shared by both waves: `w` holds, in every lane of a quad (q = lane & 3), the complete words
// i = 0..15 (per chunk) of column group (kq, j); lane q stores the words i = 4q .. 4q+3. `hi` (3-bit only)
// holds the high-plane words, complete in both lanes j and j^1; the even-j lanes store them.
// A word of which only the bits of `mask` are this launch's to write (PARTIAL: Values that leave the window token
// by token share their words with the neighbouring tokens' codes, which are already in place or still to come).
// No other lane of the launch touches the word, and launches on one cache are ordered by the caller's stream.
template <bool PARTIAL>
__device__ __forceinline__ void put_word(uint32_t* p, uint32_t v, uint32_t mask) {
  if constexpr (!PARTIAL) {
    *p = v;
  } else {
    if (mask == 0xFFFFFFFFu) *p = v;
    else if (mask != 0u) *p = (*p & ~mask) | (v & mask);
  }
}

template <int BITS, bool PARTIAL = false>
__device__ __forceinline__ void store_words(uint32_t* sec, const uint32_t (&w)[acc_words<BITS>()], const uint32_t (&hi)[16],
                                            int kq, int j, int q, uint32_t wmask = 0xFFFFFFFFu, uint32_t hmask = 0xFFFFFFFFu) {
  constexpr int kChunks = BITS == 4 ? 2 : BITS == 1 ? 0 : 1;
  constexpr int kPlane = BITS == 1 ? 0 : 256;     // first word of the 1-bit plane
#pragma unroll
  for (int c = 0; c < kChunks; c++)
#pragma unroll
    for (int n = 0; n < 4; n++) {
      const uint32_t v = q == 0 ? w[16 * c + n] : q == 1 ? w[16 * c + 4 + n] : q == 2 ? w[16 * c + 8 + n] : w[16 * c + 12 + n];
      put_word<PARTIAL>(sec + 256 * c + 4 * (16 * kq + 4 * q + n) + j, v, wmask);
    }
  if constexpr (BITS == 3 || BITS == 1) {
    if ((j & 1) == 0) {
#pragma unroll
      for (int n = 0; n < 4; n++) {
        const uint32_t v = q == 0 ? hi[n] : q == 1 ? hi[4 + n] : q == 2 ? hi[8 + n] : hi[12 + n];
        put_word<PARTIAL>(sec + kPlane + 2 * (16 * kq + 4 * q + n) + (j >> 1), v, hmask);
      }
    }
  }
}

// One workgroup of two waves quantizes and packs one (unit, 32-token tile) entirely in registers: wave 0
// the Key tile, wave 1 the Value tile. A lane owns what ends up in the same words: lane = 16*kq + 4*j + q.
//   Key wave:   q = ks; channels d0 = 32*ks + 8*kq + 2*j and d0 + 1 over the 32 tokens (two groups); a word
//               (l = 16*kq + i, j) gets its fields of slot ks + 4*m from this lane, the other ks from the quad.
//   Value wave: q = g;  tokens 8*kq + 2*j and + 1, channels 32*g .. 32*g + 31 (two groups); a word gets its
//               fields of slots 2*g, 2*g + 1 from this lane, the other blocks from the quad.
// The lanes of a quad OR their partial words together (DPP), the 1-bit plane of 3-bit codes also across the
// two j of a word; each lane then stores a quarter of the words. No LDS.
// Row r of the sequence a launch quantizes: a ring slot of the window or a row of the input.
__device__ __forceinline__ const uint16_t* source_row(const uint16_t* ring, const uint16_t* in, int64_t tok, int64_t unit_off,
                                                      const QuantArgs& a, int u, int r) {
  if (r < a.n_ring) {
    int slot = a.ring_w0 + r;
    if (slot >= a.W_cap) slot -= a.W_cap;
    return ring + ((size_t)u * a.W_cap + slot) * kD;
  }
  return in + unit_off + (int64_t)(r - a.n_ring) * tok;
}

// Row r of an ageing launch (PARTIAL): always a ring slot; the launch may span more rows than the ring has slots
// (only rows of live tokens are read).
__device__ __forceinline__ const uint16_t* ring_row(const uint16_t* ring, const QuantArgs& a, int u, int r) {
  const int slot = (a.ring_w0 + r) % a.W_cap;
  return ring + ((size_t)u * a.W_cap + slot) * kD;
}

// PARTIAL: ageing with separate fronts for Keys and Values. The Key wave works on the tiles [k_tile_a, k_tile_b)
// only; the Value wave writes the codes and metadata of the tokens [v_tok_a, v_tok_b) only, merging them into
// words that it shares with other tokens.
template <int KB, int VB, bool PARTIAL>
__global__ __launch_bounds__(128) void quantize_pack_kernel(QuantArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kq = lane >> 4, j = (lane >> 2) & 3, q = lane & 3;
  const int tile_in = blockIdx.x, jh = blockIdx.y, b = blockIdx.z;   // no integer division at the start of a short kernel
  const int u = b * a.Hkv + jh;
  if constexpr (PARTIAL) {
    const int tile_abs = a.tile0 + tile_in;
    if (wave == 0 && (tile_abs < a.k_tile_a || tile_abs >= a.k_tile_b)) return;   // wave-uniform; the waves never synchronize
  }
  uint32_t* rec = a.packed + ((size_t)u * a.tiles_cap + (size_t)(a.tile0 + tile_in)) * record_words(KB, VB);
  uint32_t hi[16];
#pragma unroll
  for (int i = 0; i < 16; i++) hi[i] = 0;

  if (wave == 0) {
    const int64_t k_off = b * a.k_unit_b + jh * a.k_unit_h;
    const int d0 = 32 * q + 8 * kq + 2 * j;
    uint32_t xw[kTile];                              // (x[tau][d0], x[tau][d0 + 1])
#pragma unroll
    for (int t = 0; t < kTile; t++) {
      const uint16_t* rowp = PARTIAL ? ring_row(a.k_ring, a, u, tile_in * kTile + t) : source_row(a.k_ring, a.k, a.k_tok, k_off, a, u, tile_in * kTile + t);
      xw[t] = *reinterpret_cast<const uint32_t*>(rowp + d0);
    }
    half2_t mn2 = as_half2(xw[0]), mx2 = mn2;
#pragma unroll
    for (int t = 1; t < kTile; t++) {
      mn2 = __builtin_elementwise_min(mn2, as_half2(xw[t]));
      mx2 = __builtin_elementwise_max(mx2, as_half2(xw[t]));
    }
    const GroupParams g0 = group_params<KB>((float)mn2[0], (float)mx2[0]);
    const GroupParams g1 = group_params<KB>((float)mn2[1], (float)mx2[1]);
    // metadata word 4*(d0/2) + f: scale pair (f = 0), minimum pair (f = 1)
    *reinterpret_cast<u32x2_t*>(rec + 4 * (d0 >> 1)) =
        u32x2_t{(uint32_t)g0.scale_h | ((uint32_t)g1.scale_h << 16), (uint32_t)g0.zero_h | ((uint32_t)g1.zero_h << 16)};
    uint32_t w[acc_words<KB>()];
#pragma unroll
    for (int i = 0; i < acc_words<KB>(); i++) w[i] = 0;
#pragma unroll
    for (int t0 = 0; t0 < kTile; t0 += 4) {
      uint32_t b0[4], b1[4];                         // biased codes of the lane's two channels
      bool near = g0.slow || g1.slow;
#pragma unroll
      for (int n = 0; n < 4; n++) {
        const half2_t xv = as_half2(xw[t0 + n]);
        b0[n] = quantize_fast<KB>(diff(xv[0], g0.mn), g0, t0 + n, near);
        b1[n] = quantize_fast<KB>(diff(xv[1], g1.mn), g1, t0 + n, near);
      }
      if (near) {
#pragma unroll
        for (int n = 0; n < 4; n++) {
          const half2_t xv = as_half2(xw[t0 + n]);
          b0[n] = quantize_exact<KB>(diff(xv[0], g0.mn), g0, t0 + n);
          b1[n] = quantize_exact<KB>(diff(xv[1], g1.mn), g1, t0 + n);
        }
      }
#pragma unroll
      for (int n = 0; n < 4; n++) {
        const int t = t0 + n;
        // the two codes side by side: the low halves of the biased codes are the codes
        const uint32_t pair = __builtin_amdgcn_perm(b1[n], b0[n], 0x05040100u);
        const int i = 4 * (t >> 3) + (t & 3), m = (t & 7) >> 2;       // word of the column group, token half
        if constexpr (KB == 1) {
          hi[i] |= pair << (8 * (j & 1) + 2 * q + m);                  // the code is the plane's bit
        } else if constexpr (KB == 4) {
          w[16 * m + i] |= pair << (4 * q);                            // chunk m, field ks
        } else {
          w[i] |= (pair & 0x00030003u) << (2 * q + 8 * m);             // slot ks + 4*m
          if constexpr (KB == 3) hi[i] |= ((pair >> 2) & 0x00010001u) << (8 * (j & 1) + 2 * q + m);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < acc_words<KB>(); i++) { w[i] |= quad_x1(w[i]); w[i] |= quad_x2(w[i]); }
    if constexpr (KB == 3 || KB == 1) {
#pragma unroll
      for (int i = 0; i < 16; i++) { hi[i] |= quad_x1(hi[i]); hi[i] |= quad_x2(hi[i]); hi[i] |= (uint32_t)__shfl_xor((int)hi[i], 4); }
    }
    store_words<KB>(rec + kMetaWords, w, hi, kq, j, q);
  } else {
    const int64_t v_off = b * a.v_unit_b + jh * a.v_unit_h;
    const int tau0 = 8 * kq + 2 * j;
    u32x4_t xr[2][4];                                // rows tau0, tau0 + 1: channels 32*q .. 32*q + 31
    // PARTIAL: which of the lane's two tokens, and of the two of lane j ^ 1, are among those that leave now
    auto leaves = [&](int tau) { const int t = (a.tile0 + tile_in) * kTile + tau; return !PARTIAL || (t >= a.v_tok_a && t < a.v_tok_b); };
    const bool mine[2] = {leaves(tau0), leaves(tau0 + 1)};
#pragma unroll
    for (int hh = 0; hh < 2; hh++)
#pragma unroll
      for (int c = 0; c < 4; c++) {
        xr[hh][c] = u32x4_t{0, 0, 0, 0};
        if (mine[hh]) {
          const uint16_t* rowp = PARTIAL ? ring_row(a.v_ring, a, u, tile_in * kTile + tau0 + hh) : source_row(a.v_ring, a.v, a.v_tok, v_off, a, u, tile_in * kTile + tau0 + hh);
          xr[hh][c] = *reinterpret_cast<const u32x4_t*>(rowp + 32 * q + 8 * c);
        }
      }
    const uint32_t wmask = (mine[0] ? 0x0000FFFFu : 0u) | (mine[1] ? 0xFFFF0000u : 0u);
    // a plane word holds the pairs j (even, bits 0-7 and 16-23) and j + 1 (bits 8-15 and 24-31); the even lane stores it
    uint32_t hmask = (mine[0] ? 0x000000FFu : 0u) | (mine[1] ? 0x00FF0000u : 0u);
    if constexpr (PARTIAL) hmask |= (leaves(tau0 + 2) ? 0x0000FF00u : 0u) | (leaves(tau0 + 3) ? 0xFF000000u : 0u);
    else hmask = 0xFFFFFFFFu;
    GroupParams gp[2];
#pragma unroll
    for (int hh = 0; hh < 2; hh++) {
      half2_t mn2 = as_half2(xr[hh][0][0]), mx2 = mn2;
#pragma unroll
      for (int e = 1; e < 16; e++) {
        mn2 = __builtin_elementwise_min(mn2, as_half2(xr[hh][e >> 2][e & 3]));
        mx2 = __builtin_elementwise_max(mx2, as_half2(xr[hh][e >> 2][e & 3]));
      }
      const float mn = fminf((float)mn2[0], (float)mn2[1]), mx = fmaxf((float)mx2[0], (float)mx2[1]);
      gp[hh] = group_params<VB>(mn, mx);
    }
    // metadata word 4*(16*g + tau0/2) + f: scale pair (f = 2), minimum pair (f = 3)
    {
      const uint32_t sc2 = (uint32_t)gp[0].scale_h | ((uint32_t)gp[1].scale_h << 16), zp2 = (uint32_t)gp[0].zero_h | ((uint32_t)gp[1].zero_h << 16);
      uint32_t* mp = rec + 4 * (16 * q + (tau0 >> 1)) + 2;
      if constexpr (!PARTIAL) {
        *reinterpret_cast<u32x2_t*>(mp) = u32x2_t{sc2, zp2};
      } else {
        put_word<true>(mp, sc2, wmask);
        put_word<true>(mp + 1, zp2, wmask);
      }
    }
    // partial words with the lane-independent shifts first (fields of slot parity e/16 and token parity hh)
    uint32_t pw[16], ph[16];
#pragma unroll
    for (int i = 0; i < 16; i++) { pw[i] = 0; ph[i] = 0; }
#pragma unroll
    for (int hh = 0; hh < 2; hh++)
#pragma unroll
      for (int e0 = 0; e0 < 32; e0 += 8) {
        uint32_t bc[8];                               // biased codes
        bool near = gp[hh].slow;
#pragma unroll
        for (int n = 0; n < 8; n++) {
          const half2_t xv = as_half2(xr[hh][e0 >> 3][n >> 1]);
          bc[n] = quantize_fast<VB>(diff(xv[n & 1], gp[hh].mn), gp[hh], e0 + n, near);
        }
        if (near) {
#pragma unroll
          for (int n = 0; n < 8; n++) {
            const half2_t xv = as_half2(xr[hh][e0 >> 3][n >> 1]);
            bc[n] = quantize_exact<VB>(diff(xv[n & 1], gp[hh].mn), gp[hh], e0 + n);
          }
        }
#pragma unroll
        for (int n = 0; n < 8; n++) {
          const int e = e0 + n;
          const int i = e & 15, sp = e >> 4;
          // fields never overflow, so the shifted biased codes are added up and the bias taken off afterwards
          if constexpr (VB == 1) {
            ph[i] += bc[n] << (16 * hh + 2 * sp);
          } else if constexpr (VB == 4) {
            pw[i] += bc[n] << (16 * hh + 4 * sp);
          } else if constexpr (VB == 2) {
            pw[i] += bc[n] << (16 * hh + 2 * sp);
          } else {
            pw[i] |= (bc[n] & 3u) << (16 * hh + 2 * sp);
            ph[i] |= ((bc[n] >> 2) & 1u) << (16 * hh + 2 * sp);
          }
        }
      }
    if constexpr (VB != 3) {
      constexpr int kField = VB == 4 ? 4 : 2;
      constexpr uint32_t kBiasSum = (kBias << 0) + (kBias << kField) + (kBias << 16) + (kBias << (16 + kField));
#pragma unroll
      for (int i = 0; i < 16; i++) {
        if constexpr (VB == 1) ph[i] -= kBiasSum; else pw[i] -= kBiasSum;
      }
    }
    uint32_t w[acc_words<VB>()];
    if constexpr (VB == 4) {
      // slot 2*g + sp: chunk g/2, field 2*(g%2) + sp; the chunk's words are complete after the pair (g, g^1)
#pragma unroll
      for (int i = 0; i < 16; i++) {
        uint32_t v = pw[i] << (8 * (q & 1));
        v |= quad_x1(v);
        const uint32_t other = quad_x2(v);            // the other chunk's words, from lane g ^ 2
        w[i] = (q & 2) ? other : v;                  // chunk 0
        w[16 + i] = (q & 2) ? v : other;             // chunk 1
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; i++) {
        w[i] = pw[i] << (4 * q);
        w[i] |= quad_x1(w[i]); w[i] |= quad_x2(w[i]);
      }
      if constexpr (VB == 3 || VB == 1) {
        // bit plane: bit 16*hh + 8*(j%2) + 2*(slot%4) + slot/4 with slot = 2*g + sp
#pragma unroll
        for (int i = 0; i < 16; i++) {
          hi[i] = ph[i] << (8 * (j & 1) + 4 * (q & 1) + (q >> 1));
          hi[i] |= quad_x1(hi[i]); hi[i] |= quad_x2(hi[i]); hi[i] |= (uint32_t)__shfl_xor((int)hi[i], 4);
        }
      }
    }
    store_words<VB, PARTIAL>(rec + kMetaWords + tile_words(KB), w, hi, kq, j, q, wmask, hmask);
  }
}

// x = code * s_i + min, evaluated in fp32 (multiply, then add), of the first n_tokens tokens of every unit.
__global__ __launch_bounds__(256) void dequant_kernel(DequantArgs a) {
  const int u = blockIdx.y, tile_i = blockIdx.x;
  const uint32_t* rec = a.packed + ((size_t)u * a.tiles_cap + tile_i) * record_words(a.k_bits, a.v_bits);
  for (int e = threadIdx.x; e < kTile * kD; e += blockDim.x) {
    const int tau = e / kD, d = e % kD;
    const int t = tile_i * kTile + tau;
    if (t < a.n_tokens) a.out[((size_t)u * a.n_tokens + t) * kD + d] = dequant_elem(rec, a.k_bits, a.v_bits, a.which, tau, d);
  }
}

// New tokens of every unit into consecutive ring slots of the two fp16 windows (one full row each).
__global__ __launch_bounds__(128) void append_kernel(AppendArgs a) {
  const int u = blockIdx.x, i = blockIdx.y, d = threadIdx.x;
  const int64_t src = (int64_t)(u / a.Hkv) * a.batch + (int64_t)(u % a.Hkv) * a.head + (int64_t)i * a.tok + d;
  const size_t dst = ((size_t)u * a.W_cap + (a.slot + i) % a.W_cap) * kD + d;
  a.k_win[dst] = a.k_new[src];
  a.v_win[dst] = a.v_new[src];
}

// Load-only pass over a buffer in the launch shape of the attention kernel (one workgroup per contiguous span,
// 16 bytes per lane and load, non-temporal policy, four loads in flight per lane): the rate a kernel of this
// shape can reach on the machine at hand when it does nothing but read.
__global__ __launch_bounds__(768) void stream_read_kernel(const u32x4_t* buf, size_t n16, uint32_t* sink) {
  const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t begin = (size_t)blockIdx.x * per_wg;
  const size_t end = begin + per_wg < n16 ? begin + per_wg : n16;
  const size_t step = blockDim.x;
  u32x4_t acc = {0, 0, 0, 0};
  size_t i = begin + threadIdx.x;
  for (; i + 3 * step < end; i += 4 * step) {
    const u32x4_t a = __builtin_nontemporal_load(buf + i), b = __builtin_nontemporal_load(buf + i + step);
    const u32x4_t c = __builtin_nontemporal_load(buf + i + 2 * step), d = __builtin_nontemporal_load(buf + i + 3 * step);
    acc |= (a ^ b) | (c ^ d);
  }
  for (; i < end; i += step) acc |= __builtin_nontemporal_load(buf + i);
  // never true for real data in all four words at once: keeps the loads alive without a store per lane
  if ((acc[0] & acc[1] & acc[2] & acc[3]) == 0xFFFFFFFFu && sink) sink[0] = 1u;
}

template <int KB, int VB, bool PARTIAL>
hipError_t launch_qp(const QuantArgs& a, dim3 grid, hipStream_t s) {
  quantize_pack_kernel<KB, VB, PARTIAL><<<grid, 128, 0, s>>>(a);
  return hipGetLastError();
}

// The bit pairs the library accepts: every pair of 1..4 (a 16-bit side never reaches the quantizer).
template <bool PARTIAL>
hipError_t launch_bits(const QuantArgs& a, int k_bits, int v_bits, int n_tiles, int units, hipStream_t s) {
  if (n_tiles == 0 || units == 0) return hipSuccess;
  const dim3 grid(n_tiles, a.Hkv, units / a.Hkv);
  switch (k_bits * 10 + v_bits) {
    case 11: return launch_qp<1, 1, PARTIAL>(a, grid, s);
    case 12: return launch_qp<1, 2, PARTIAL>(a, grid, s);
    case 13: return launch_qp<1, 3, PARTIAL>(a, grid, s);
    case 14: return launch_qp<1, 4, PARTIAL>(a, grid, s);
    case 21: return launch_qp<2, 1, PARTIAL>(a, grid, s);
    case 22: return launch_qp<2, 2, PARTIAL>(a, grid, s);
    case 23: return launch_qp<2, 3, PARTIAL>(a, grid, s);
    case 24: return launch_qp<2, 4, PARTIAL>(a, grid, s);
    case 31: return launch_qp<3, 1, PARTIAL>(a, grid, s);
    case 32: return launch_qp<3, 2, PARTIAL>(a, grid, s);
    case 33: return launch_qp<3, 3, PARTIAL>(a, grid, s);
    case 34: return launch_qp<3, 4, PARTIAL>(a, grid, s);
    case 41: return launch_qp<4, 1, PARTIAL>(a, grid, s);
    case 42: return launch_qp<4, 2, PARTIAL>(a, grid, s);
    case 43: return launch_qp<4, 3, PARTIAL>(a, grid, s);
    case 44: return launch_qp<4, 4, PARTIAL>(a, grid, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_quantize_pack(const QuantArgs& a, int k_bits, int v_bits, int n_tiles, int units, hipStream_t s) {
  return launch_bits<false>(a, k_bits, v_bits, n_tiles, units, s);
}

hipError_t launch_quantize_fronts(const QuantArgs& a, int k_bits, int v_bits, int n_tiles, int units, hipStream_t s) {
  return launch_bits<true>(a, k_bits, v_bits, n_tiles, units, s);
}

hipError_t launch_dequant(const DequantArgs& a, int units, hipStream_t s) {
  if (a.n_tokens == 0 || units == 0) return hipSuccess;
  dequant_kernel<<<dim3((a.n_tokens + kTile - 1) / kTile, units), 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* buf, size_t bytes, int workgroups, int threads, uint32_t* sink, hipStream_t s) {
  if (bytes < 16 || workgroups < 1) return hipSuccess;
  stream_read_kernel<<<workgroups, threads, 0, s>>>(reinterpret_cast<const u32x4_t*>(buf), bytes / 16, sink);
  return hipGetLastError();
}

hipError_t launch_append(const AppendArgs& a, hipStream_t s) {
  if (a.n == 0 || a.units == 0) return hipSuccess;
  append_kernel<<<dim3(a.units, a.n), 128, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace kvmix
