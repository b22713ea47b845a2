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

constexpr int kRow = kD + 8;  // LDS row pitch in fp16 elements (272 B) to spread banks

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

// One group of 32 values (already in registers as fp32, exact images of fp16 inputs).
template <int BITS>
__device__ __forceinline__ void quantize_group(const float (&x)[32], uint8_t (&code)[32], uint16_t& scale_h, uint16_t& zero_h) {
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int i = 1; i < 32; i++) {
    mn = x[i] < mn ? x[i] : mn;
    mx = x[i] > mx ? x[i] : mx;
  }
  if (mn == 0.0f) mn = 0.0f;                      // -0 -> +0
  const float range = mx - mn;
  const float s32 = range / (float)((1 << BITS) - 1);
  const half_t sh = (half_t)s32;                  // round-to-nearest-even
  const float s = (float)sh;
  scale_h = __builtin_bit_cast(uint16_t, sh);
  zero_h = __builtin_bit_cast(uint16_t, (half_t)mn);
#pragma unroll
  for (int i = 0; i < 32; i++) {
    float r = 0.0f;
    if (s != 0.0f) {
      const float t = (x[i] - mn) / step_of<BITS>(s, i);
      r = __builtin_rintf(t);
      const float hi = (float)qmax_of<BITS>(i);
      r = r < 0.0f ? 0.0f : r;
      r = r > hi ? hi : r;
    }
    code[i] = (uint8_t)r;
  }
}

// Assemble and store the words of one tile from the code bytes in LDS.
template <int BITS, bool IS_VALUE>
__device__ __forceinline__ void pack_tile(const uint8_t* cs /*[32][128]*/, uint32_t* dst, int tid, int nthreads) {
  constexpr int kLoWords = (BITS == 4) ? 512 : 256;
  for (int w = tid; w < kLoWords; w += nthreads) {
    const int chunk = w >> 8, rem = w & 255, l = rem >> 2, j = rem & 3;
    uint32_t val = 0;
#pragma unroll
    for (int hh = 0; hh < 2; hh++) {
      if (BITS == 4) {
#pragma unroll
        for (int f = 0; f < 4; f++) {
          int tau, d;
          if (IS_VALUE) value_td(l, j, hh, 4 * chunk + f, tau, d); else key_td(l, j, hh, 4 * chunk + f, tau, d);
          val |= (uint32_t)cs[tau * kD + d] << (16 * hh + 4 * f);
        }
      } else {
#pragma unroll
        for (int slot = 0; slot < 8; slot++) {
          int tau, d;
          if (IS_VALUE) value_td(l, j, hh, slot, tau, d); else key_td(l, j, hh, slot, tau, d);
          val |= (uint32_t)(cs[tau * kD + d] & 3) << (16 * hh + 2 * slot);
        }
      }
    }
    dst[w] = val;
  }
  if (BITS == 3) {
    for (int w = tid; w < 128; w += nthreads) {
      const int l = w >> 1, jp = w & 1;
      uint32_t val = 0;
#pragma unroll
      for (int jj = 0; jj < 2; jj++)
#pragma unroll
        for (int hh = 0; hh < 2; hh++)
#pragma unroll
          for (int slot = 0; slot < 8; slot++) {
            int tau, d;
            if (IS_VALUE) value_td(l, 2 * jp + jj, hh, slot, tau, d); else key_td(l, 2 * jp + jj, hh, slot, tau, d);
            val |= (uint32_t)(cs[tau * kD + d] >> 2) << (16 * hh + 8 * jj + 2 * (slot & 3) + (slot >> 2));
          }
      dst[256 + w] = val;
    }
  }
}

// One workgroup (256 threads) quantizes and packs the Key tile and the Value tile of one
// (unit, 32-token tile): waves 0-1 own the 128 Key groups (one channel each), waves 2-3 the
// 128 Value groups (one (token, 32-channel block) each).
template <int KB, int VB>
__global__ __launch_bounds__(256) void quantize_pack_kernel(QuantArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t xs[2][kTile * kRow];
  __shared__ __attribute__((aligned(16))) uint8_t cs[2][kTile * kD];
  const int tid = threadIdx.x;
  const int tile_in = blockIdx.x, u = blockIdx.y;
  const int b = u / a.Hkv, jh = u % a.Hkv;
  const uint16_t* kin = a.k + b * a.k_unit_b + jh * a.k_unit_h + (int64_t)tile_in * kTile * a.k_tok;
  const uint16_t* vin = a.v + b * a.v_unit_b + jh * a.v_unit_h + (int64_t)tile_in * kTile * a.v_tok;

  // stage the two fp16 tiles in LDS with 16-byte loads
#pragma unroll
  for (int p = 0; p < 2; p++) {
    const int tau = (tid >> 4) + 16 * p, dc = (tid & 15) * 8;
    const u32x4_t kv = *reinterpret_cast<const u32x4_t*>(kin + (int64_t)tau * a.k_tok + dc);
    *reinterpret_cast<u32x4_t*>(&xs[0][tau * kRow + dc]) = kv;
    const u32x4_t vv = *reinterpret_cast<const u32x4_t*>(vin + (int64_t)tau * a.v_tok + dc);
    *reinterpret_cast<u32x4_t*>(&xs[1][tau * kRow + dc]) = vv;
  }
  __syncthreads();

  uint32_t* rec = a.packed + ((size_t)u * a.tiles_cap + (size_t)(a.tile0 + tile_in)) * record_words(KB, VB);
  uint16_t* meta = reinterpret_cast<uint16_t*>(rec);
  float x[32];
  uint8_t code[32];
  uint16_t sh, zh;
  if (tid < 128) {
    const int d = tid;  // Key group: channel d, tokens 0..31
#pragma unroll
    for (int t = 0; t < 32; t++) x[t] = (float)__builtin_bit_cast(half_t, xs[0][t * kRow + d]);
    quantize_group<KB>(x, code, sh, zh);
#pragma unroll
    for (int t = 0; t < 32; t++) cs[0][t * kD + d] = code[t];
    meta[key_meta_half(d, 0)] = sh;
    meta[key_meta_half(d, 1)] = zh;
  } else {
    const int tau = (tid - 128) & 31, g = (tid - 128) >> 5;  // Value group: token tau, channels 32g..32g+31
#pragma unroll
    for (int c = 0; c < 4; c++) {
      const u32x4_t vv = *reinterpret_cast<const u32x4_t*>(&xs[1][tau * kRow + 32 * g + 8 * c]);
      const uint16_t* e = reinterpret_cast<const uint16_t*>(&vv);
#pragma unroll
      for (int t = 0; t < 8; t++) x[8 * c + t] = (float)__builtin_bit_cast(half_t, e[t]);
    }
    quantize_group<VB>(x, code, sh, zh);
#pragma unroll
    for (int c = 0; c < 8; c++) {
      uint32_t w = (uint32_t)code[4 * c] | ((uint32_t)code[4 * c + 1] << 8) | ((uint32_t)code[4 * c + 2] << 16) | ((uint32_t)code[4 * c + 3] << 24);
      *reinterpret_cast<uint32_t*>(&cs[1][tau * kD + 32 * g + 4 * c]) = w;
    }
    meta[value_meta_half(tau, g, 0)] = sh;
    meta[value_meta_half(tau, g, 1)] = zh;
  }
  __syncthreads();

  pack_tile<KB, false>(cs[0], rec + kMetaWords, tid, 256);
  pack_tile<VB, true>(cs[1], rec + kMetaWords + tile_words(KB), tid, 256);
}

// x = code * s_i + min, evaluated in fp32 (multiply, then add).
__global__ __launch_bounds__(256) void dequant_kernel(DequantArgs a) {
  const int u = blockIdx.y, tile_i = blockIdx.x;
  const uint32_t* rec = a.packed + ((size_t)u * a.tiles_cap + tile_i) * record_words(a.k_bits, a.v_bits);
  const uint16_t* meta = reinterpret_cast<const uint16_t*>(rec);
  const int bits = a.which ? a.v_bits : a.k_bits;
  const uint32_t* words = rec + kMetaWords + (a.which ? tile_words(a.k_bits) : 0);
  for (int e = threadIdx.x; e < kTile * kD; e += blockDim.x) {
    const int tau = e / kD, d = e % kD;
    int l, j, hh, slot, gi, ms, mz;
    if (a.which == 0) {
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
    a.out[((size_t)u * a.n_tiles + tile_i) * kTile * kD + e] = prod + mn;
  }
}

// New token of every unit into ring slot `slot` of the two fp16 windows.
__global__ __launch_bounds__(128) void append_kernel(AppendArgs a) {
  const int u = blockIdx.x, d = threadIdx.x;
  a.k_win[((size_t)u * a.W_cap + a.slot) * kD + d] = a.k_new[(size_t)u * kD + d];
  a.v_win[((size_t)u * a.W_cap + a.slot) * kD + d] = a.v_new[(size_t)u * kD + d];
}

template <int KB, int VB>
hipError_t launch_qp(const QuantArgs& a, dim3 grid, hipStream_t s) {
  quantize_pack_kernel<KB, VB><<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize_pack(const QuantArgs& a, int k_bits, int v_bits,
                                int n_tiles, int units, hipStream_t s) {
  if (n_tiles == 0 || units == 0) return hipSuccess;
  const dim3 grid(n_tiles, units);
  switch (k_bits * 10 + v_bits) {
    case 22: return launch_qp<2, 2>(a, grid, s);
    case 23: return launch_qp<2, 3>(a, grid, s);
    case 24: return launch_qp<2, 4>(a, grid, s);
    case 32: return launch_qp<3, 2>(a, grid, s);
    case 33: return launch_qp<3, 3>(a, grid, s);
    case 34: return launch_qp<3, 4>(a, grid, s);
    case 42: return launch_qp<4, 2>(a, grid, s);
    case 43: return launch_qp<4, 3>(a, grid, s);
    case 44: return launch_qp<4, 4>(a, grid, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_dequant(const DequantArgs& a, int units, hipStream_t s) {
  if (a.n_tiles == 0 || units == 0) return hipSuccess;
  dequant_kernel<<<dim3(a.n_tiles, units), 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_append(const AppendArgs& a, hipStream_t s) {
  append_kernel<<<a.units, 128, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace kvmix
