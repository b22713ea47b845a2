// Fused decode attention over the packed mixed-bit KV cache plus the fp16 recent window (gfx950).
//
// Paper Sec. 3.4 item 2 (dequantize on the fly while multiplying, never materialize fp16 K/V),
// Sec. 3.2.2 step 4 (x = q*s + min), Sec. 3.3 (recent tokens stay in full precision).
//
// Formulation. For one kv head and one 32-token tile
//   score[t][h] = sum_d code[t][d] * (q[h][d]*s[d])  +  sum_d q[h][d]*z[d]
//   out[d][h]  += sum_t code[t][d] * (p[t][h]*s[t][g(d)])  +  sum_t p[t][h]*z[t][g(d)]
// Both code sums are 16x16x32 fp16 MFMAs whose A operand is the packed word ANDed with a mask:
// a 2/4-bit field left in place inside a zero fp16 pattern is the subnormal code * 2^(pos-24),
// exact, and MFMA honours subnormal inputs. The scale factors ride in the B operand, split
// into an fp16 (hi, lo) pair held in two MFMA columns so that the products stay exact to
// ~22 bits; the up-to-8 query heads of the group use columns 0..7 (hi) and 8..15 (lo).
// The zero-point sums and the fp16 window are MFMAs on plain fp16 operands. Softmax is online,
// per wave, with a lazily raised reference maximum; waves of a workgroup take tiles from a
// shared counter and merge through LDS; splits of one unit merge through a workspace, the last
// arriving workgroup writes the output.
#include "kvmix_common.hpp"

namespace kvmix {

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * kWave;
constexpr float kRefMargin = 4.0f;   // reference maximum is raised to (tile max + margin), log2 units

__device__ __forceinline__ float4_t mfma16(half8_t a, half8_t b, float4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
// value of lane (l ^ 8) within each row of 16 lanes
__device__ __forceinline__ float ror8(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false));
}
__device__ __forceinline__ half8_t as_half8(u32x4_t v) { return __builtin_bit_cast(half8_t, v); }

// bit position (inside a 16-bit half, after the unpack shift) of the field that feeds slot
// `s` (0..3 = slot % 4): the MFMA sees code * 2^(pos - 24).
template <int BITS> __device__ __forceinline__ constexpr int field_pos(int s) { return BITS == 4 ? 4 * (s & 1) : 2 * s; }

// ---- A operands from packed words. w: the lane's words of the code plane(s).
// 2-bit plane (also the low plane of 3-bit): 4 words, slot field at bits 2*slot of each half.
__device__ __forceinline__ half8_t unpack2(const u32x4_t& w, const u32x4_t& w8, int slot) {
  const uint32_t mask = 0x00030003u << (2 * (slot & 3));
  const u32x4_t src = (slot & 4) ? w8 : w;
  return as_half8(src & mask);
}
// 4-bit: 8 words (two chunks of 4), slot -> chunk slot/4, field slot%4 at bits 4*field.
__device__ __forceinline__ half8_t unpack4(const u32x4_t& w, const u32x4_t& w8, int field) {
  const uint32_t mask = 0x000F000Fu << (4 * (field & 1));
  const u32x4_t src = (field & 2) ? w8 : w;
  return as_half8(src & mask);
}
// 1-bit high plane of 3-bit codes: 2 words; word j/2 holds, for pair j, bit 8*(j%2) + 2*(slot%4) + slot/4.
// hs[v] = plane shifted so that variant v = 2*(j%2) + slot/4 has its bits at 2*(slot%4) + 2.
__device__ __forceinline__ half8_t unpack1(const u32x2_t (&hs)[4], int slot) {
  const uint32_t mask = 0x00010001u << (2 * (slot & 3) + 2);
  const int hi = slot >> 2;
  u32x4_t r;
  r[0] = hs[0 + hi][0] & mask;   // j = 0: word 0, variant (0, hi)
  r[1] = hs[2 + hi][0] & mask;   // j = 1: word 0, variant (1, hi)
  r[2] = hs[0 + hi][1] & mask;   // j = 2: word 1
  r[3] = hs[2 + hi][1] & mask;   // j = 3: word 1
  return as_half8(r);
}
__device__ __forceinline__ void shift_hi_plane(const u32x2_t& h, u32x2_t (&hs)[4]) {
  hs[0] = h << 2;   // (j%2 = 0, slot/4 = 0): source bit 2*s     -> 2*s + 2
  hs[1] = h << 1;   // (0, 1):                 source bit 2*s + 1 -> 2*s + 2
  hs[2] = h >> 6;   // (1, 0):                 source bit 2*s + 8 -> 2*s + 2
  hs[3] = h >> 7;   // (1, 1):                 source bit 2*s + 9 -> 2*s + 2
}

template <int BITS> struct Codes;   // the lane's share of one packed tile
template <> struct Codes<2> {
  u32x4_t w, w8;
  __device__ __forceinline__ void load(const uint32_t* tile, int lane) {
    w = *reinterpret_cast<const u32x4_t*>(tile + 4 * lane);
  }
  __device__ __forceinline__ void prep() { w8 = w >> 8; }
  __device__ __forceinline__ half8_t lo(int slot) const { return unpack2(w, w8, slot); }
};
template <> struct Codes<3> {
  u32x4_t w, w8; u32x2_t h; u32x2_t hs[4];
  __device__ __forceinline__ void load(const uint32_t* tile, int lane) {
    w = *reinterpret_cast<const u32x4_t*>(tile + 4 * lane);
    h = *reinterpret_cast<const u32x2_t*>(tile + 256 + 2 * lane);
  }
  __device__ __forceinline__ void prep() { w8 = w >> 8; shift_hi_plane(h, hs); }
  __device__ __forceinline__ half8_t lo(int slot) const { return unpack2(w, w8, slot); }
  __device__ __forceinline__ half8_t hi(int slot) const { return unpack1(hs, slot); }
};
template <> struct Codes<4> {
  u32x4_t w[2], w8[2];
  __device__ __forceinline__ void load(const uint32_t* tile, int lane) {
    w[0] = *reinterpret_cast<const u32x4_t*>(tile + 4 * lane);
    w[1] = *reinterpret_cast<const u32x4_t*>(tile + 256 + 4 * lane);
  }
  __device__ __forceinline__ void prep() { w8[0] = w[0] >> 8; w8[1] = w[1] >> 8; }
  __device__ __forceinline__ half8_t lo(int slot) const { return unpack4(w[slot >> 2], w8[slot >> 2], slot & 3); }
};

// fp32 value -> the lane's part of its fp16 (hi, lo) split
__device__ __forceinline__ half_t split_part(float x, bool lo_part) {
  const half_t hi = (half_t)x;
  const half_t lo = (half_t)(x - (float)hi);
  return lo_part ? lo : hi;
}

template <int KB, int VB, int G>
__global__ __launch_bounds__(kThreads) void decode_attn_kernel(AttnArgs a) {
  __shared__ int s_next;
  __shared__ int s_last;
  __shared__ float red_o[kWaves][G][kD];
  __shared__ float red_m[kWaves][G];
  __shared__ float red_l[kWaves][G];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, kq = lane >> 4;         // MFMA column / row index, k-quarter
  const int h = col & 7;
  const bool lo_part = col >= 8;
  const bool col_valid = h < G;
  const int sp = blockIdx.x, u = blockIdx.y;
  const int b = u / a.Hkv, jh = u % a.Hkv;

  const int n_wt = a.W_cap / kTile;
  const int n_items = n_wt + a.n_tiles;
  const int item_begin = (int)(((long long)sp * n_items) / a.n_splits);
  const int item_end = (int)(((long long)(sp + 1) * n_items) / a.n_splits);
  if (tid == 0) s_next = item_begin;
  __syncthreads();

  // query operands: B columns hold q of head h in the hi column, zero elsewhere
  half8_t qB[4];
  float qf[4][8];    // fp32 q, prescaled by 2^-field_pos for the code products
  {
    const uint16_t* qp = a.q + ((size_t)b * a.Hq + (size_t)jh * G + h) * kD;
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      half8_t v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (col_valid) v = *reinterpret_cast<const half8_t*>(qp + 32 * ks + 8 * kq);
#pragma unroll
      for (int e = 0; e < 8; e++) qf[ks][e] = (float)v[e] * __builtin_ldexpf(1.0f, -field_pos<KB>(ks));
      const half8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
      qB[ks] = lo_part ? zero8 : v;
    }
  }

  const float c_code = a.scale_log2 * 16777216.0f;   // code products carry 2^-24
  const float c_plain = a.scale_log2;

  float4_t acc[8];
  float4_t accZ = {0, 0, 0, 0};
#pragma unroll
  for (int m = 0; m < 8; m++) acc[m] = float4_t{0, 0, 0, 0};
  float mref = -INFINITY, lsum = 0.0f;

  const size_t tile_base = (size_t)u * a.tiles_cap;

  for (;;) {
    int item = 0;
    if (lane == 0) item = atomicAdd(&s_next, 1);
    item = __builtin_amdgcn_readfirstlane(item);
    if (item >= item_end) break;

    float x[8];            // log2-domain scores of tokens 8*kq + e of this tile, column col
    const bool is_window = item < n_wt;
    int slot0 = 0;
    size_t tile = 0;

    if (is_window) {
      slot0 = item * kTile;
      // validity of the lane's 8 slots in the ring
      bool any_valid = false;
      {
        const int first = (slot0 - a.w0 + a.W_cap) % a.W_cap;   // ring rank of the tile's first slot
        any_valid = first < a.n_w;                               // w0 and tiles are 32-aligned
      }
      if (!any_valid) continue;
      const uint16_t* kw = a.k_win + ((size_t)u * a.W_cap + slot0) * kD;
      float4_t S[2] = {float4_t{0, 0, 0, 0}, float4_t{0, 0, 0, 0}};
#pragma unroll
      for (int m = 0; m < 2; m++) {
        const int tau = 8 * (col >> 2) + 4 * m + (col & 3);   // row `col` of M-tile m
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
          const half8_t A = *reinterpret_cast<const half8_t*>(kw + (size_t)tau * kD + 32 * ks + 8 * kq);
          S[m] = mfma16(A, qB[ks], S[m]);
        }
      }
#pragma unroll
      for (int m = 0; m < 2; m++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int rank = (slot0 + 8 * kq + 4 * m + r - a.w0 + a.W_cap) % a.W_cap;
          const float xv = S[m][r] * c_plain;
          x[4 * m + r] = rank < a.n_w ? xv : -INFINITY;
        }
    } else {
      tile = tile_base + (size_t)(item - n_wt);
      Codes<KB> kc;
      kc.load(a.k_codes + tile * tile_words(KB), lane);
      kc.prep();
      // scale-folded query (hi | lo part per column) and zero-point term
      half8_t Bk[4];
      float4_t Sz = {0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        const half8_t s8 = *reinterpret_cast<const half8_t*>(a.k_scale + tile * kD + 32 * ks + 8 * kq);
        const half8_t z8 = *reinterpret_cast<const half8_t*>(a.k_zero + tile * kD + 32 * ks + 8 * kq);
#pragma unroll
        for (int e = 0; e < 8; e++) Bk[ks][e] = split_part(qf[ks][e] * (float)s8[e], lo_part);
        Sz = mfma16(z8, qB[ks], Sz);     // every A row is the zero-point vector
      }
      float4_t S[2] = {float4_t{0, 0, 0, 0}, float4_t{0, 0, 0, 0}};
#pragma unroll
      for (int m = 0; m < 2; m++)
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
          S[m] = mfma16(kc.lo(ks + 4 * m), Bk[ks], S[m]);
          if constexpr (KB == 3) S[m] = mfma16(kc.hi(ks + 4 * m), Bk[ks], S[m]);
        }
      if constexpr (KB == 3) {   // tokens 10 and 21 of the group step by s*7/3
        if (kq == 1) S[0][2] *= (7.0f / 3.0f);
        if (kq == 2) S[1][1] *= (7.0f / 3.0f);
      }
      const float zt = Sz[0] * c_plain;
#pragma unroll
      for (int m = 0; m < 2; m++)
#pragma unroll
        for (int r = 0; r < 4; r++) x[4 * m + r] = S[m][r] * c_code + zt;
    }
    // hi column + lo column -> full score in both lanes
#pragma unroll
    for (int e = 0; e < 8; e++) x[e] = x[e] + ror8(x[e]);

    // online softmax with a lazily raised reference
    float mx = x[0];
#pragma unroll
    for (int e = 1; e < 8; e++) mx = fmaxf(mx, x[e]);
    if (__any(mx > mref)) {
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = mx > mref ? mx + kRefMargin : mref;
      const float f = (mnew == mref) ? 1.0f : __builtin_exp2f(mref - mnew);
      mref = mnew;
      lsum *= f;
      accZ *= f;
#pragma unroll
      for (int m = 0; m < 8; m++) acc[m] *= f;
    }
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
      p[e] = col_valid ? __builtin_exp2f(x[e] - mref) : 0.0f;
      lsum += p[e];
    }
    half8_t PB;
#pragma unroll
    for (int e = 0; e < 8; e++) PB[e] = split_part(p[e], lo_part);

    if (is_window) {
      const uint16_t* vw = a.v_win + (size_t)u * kD * a.W_cap + slot0 + 8 * kq;
#pragma unroll
      for (int m = 0; m < 8; m++) {
        half8_t A = *reinterpret_cast<const half8_t*>(vw + (size_t)(16 * m + col) * a.W_cap);
        float4_t t = mfma16(A, PB, float4_t{0, 0, 0, 0});
        if constexpr (VB == 3) {   // the final 7/3 step factor of channels 10 / 21 applies to codes only
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int dd = 16 * (m & 1) + 4 * kq + r;
            if (dd == 10 || dd == 21) t[r] *= (3.0f / 7.0f);
          }
        }
        acc[m] += t * __builtin_ldexpf(1.0f, field_pos<VB>(m & 3) - 24);
      }
    } else {
      Codes<VB> vc;
      vc.load(a.v_codes + tile * tile_words(VB), lane);
      vc.prep();
      half8_t Bv[4];
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const half8_t s8 = *reinterpret_cast<const half8_t*>(a.v_scale + tile * kD + 32 * g + 8 * kq);
#pragma unroll
        for (int e = 0; e < 8; e++) Bv[g][e] = split_part(p[e] * (float)s8[e], lo_part);
      }
      // zero-point term: A row i carries the zero-points of channel block i % 4
      const half8_t z8 = *reinterpret_cast<const half8_t*>(a.v_zero + tile * kD + 32 * (col & 3) + 8 * kq);
      accZ = mfma16(z8, PB, accZ);
#pragma unroll
      for (int m = 0; m < 8; m++) {
        acc[m] = mfma16(vc.lo(m), Bv[m >> 1], acc[m]);
        if constexpr (VB == 3) acc[m] = mfma16(vc.hi(m), Bv[m >> 1], acc[m]);
      }
    }
  }

  // ---- per-wave result: undo the field scaling, add hi and lo columns, add the zero-point term
  lsum += __shfl_xor(lsum, 16);
  lsum += __shfl_xor(lsum, 32);
#pragma unroll
  for (int m = 0; m < 8; m++) {
    const float sc = __builtin_ldexpf(1.0f, 24 - field_pos<VB>(m & 3));
#pragma unroll
    for (int r = 0; r < 4; r++) {
      float v = acc[m][r] * sc;
      if (VB == 3) {   // channels 10 and 21 of each block of 32 step by s*7/3
        const int dd = 16 * (m & 1) + 4 * kq + r;
        if (dd == 10 || dd == 21) v *= (7.0f / 3.0f);
      }
      v += accZ[(m >> 1)];          // row 4*kq' + r of accZ is channel block r: pick block m/2
      v += ror8(v);
      if (col < G) red_o[wave][col][16 * m + 4 * kq + r] = v;
    }
  }
  if (col < G && kq == 0) { red_m[wave][col] = mref; red_l[wave][col] = lsum; }
  __syncthreads();

  for (int idx = tid; idx < G * kD; idx += kThreads) {
    const int hh = idx / kD, d = idx % kD;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; w++) M = fmaxf(M, red_m[w][hh]);
    float L = 0.0f, O = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; w++) {
      const float mw = red_m[w][hh];
      const float f = (mw == -INFINITY) ? 0.0f : __builtin_exp2f(mw - M);
      L += red_l[w][hh] * f;
      O += red_o[w][hh][d] * f;
    }
    if (a.n_splits == 1) {
      a.out[((size_t)b * a.Hq + (size_t)jh * G + hh) * kD + d] = __builtin_bit_cast(uint16_t, (half_t)(O / L));
    } else {
      float* pp = a.part + (((size_t)u * a.n_splits + sp) * G + hh) * (kD + 2);
      if (d == 0) { pp[0] = M; pp[1] = L; }
      pp[2 + d] = O;
    }
  }
  if (a.n_splits == 1) return;

  // ---- split merge: the last workgroup of the unit to arrive combines all partials
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const uint32_t prev = atomicAdd(&a.counters[u], 1u);
    s_last = (prev == (uint32_t)a.n_splits - 1u);
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  for (int idx = tid; idx < G * kD; idx += kThreads) {
    const int hh = idx / kD, d = idx % kD;
    const float* base = a.part + ((size_t)u * a.n_splits * G + hh) * (kD + 2);
    const size_t stride = (size_t)G * (kD + 2);
    float M = -INFINITY;
    for (int s = 0; s < a.n_splits; s++) M = fmaxf(M, __builtin_nontemporal_load(base + s * stride));
    float L = 0.0f, O = 0.0f;
    for (int s = 0; s < a.n_splits; s++) {
      const float ms = __builtin_nontemporal_load(base + s * stride);
      const float f = (ms == -INFINITY) ? 0.0f : __builtin_exp2f(ms - M);
      L += __builtin_nontemporal_load(base + s * stride + 1) * f;
      O += __builtin_nontemporal_load(base + s * stride + 2 + d) * f;
    }
    a.out[((size_t)b * a.Hq + (size_t)jh * G + hh) * kD + d] = __builtin_bit_cast(uint16_t, (half_t)(O / L));
  }
  if (tid == 0) a.counters[u] = 0;
}

template <int KB, int VB>
hipError_t launch_g(const AttnArgs& a, int G, dim3 grid, hipStream_t s) {
  switch (G) {
    case 1: decode_attn_kernel<KB, VB, 1><<<grid, kThreads, 0, s>>>(a); break;
    case 2: decode_attn_kernel<KB, VB, 2><<<grid, kThreads, 0, s>>>(a); break;
    case 4: decode_attn_kernel<KB, VB, 4><<<grid, kThreads, 0, s>>>(a); break;
    case 8: decode_attn_kernel<KB, VB, 8><<<grid, kThreads, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

int attn_threads() { return kThreads; }

hipError_t launch_decode_attn(const AttnArgs& a, int k_bits, int v_bits, int G, int units, hipStream_t s) {
  const dim3 grid(a.n_splits, units);
  switch (k_bits * 10 + v_bits) {
    case 22: return launch_g<2, 2>(a, G, grid, s);
    case 23: return launch_g<2, 3>(a, G, grid, s);
    case 24: return launch_g<2, 4>(a, G, grid, s);
    case 32: return launch_g<3, 2>(a, G, grid, s);
    case 33: return launch_g<3, 3>(a, G, grid, s);
    case 34: return launch_g<3, 4>(a, G, grid, s);
    case 42: return launch_g<4, 2>(a, G, grid, s);
    case 43: return launch_g<4, 3>(a, G, grid, s);
    case 44: return launch_g<4, 4>(a, G, grid, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace kvmix
