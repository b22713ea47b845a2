// Decode attention over the tokens that lie between the Key front and the Value front of a cache whose Keys and
// Values age separately (paper Sec. 3.3: the Recent Pivotal Context ratio of a layer's Keys and of its Values may
// differ; Sec. 3.2.2 step 4 for the dequantization).
//
// The main attention kernel works on tiles whose Keys and Values are both packed and on window tiles whose Keys and
// Values are both fp16. The tokens in between ((r_k - r_v) x context of them under the count formula) have one
// side packed and the other in the ring, and the Value front may stand inside a tile. This kernel takes them tile by
// tile: a wave turns the tile's Key rows into fp32 in its own LDS area (from the packed record: every lane unpacks
// the 64 codes of its 16-byte column, x = code * s_i + min; or from the fp16 ring), takes the scores and the softmax
// numerators on the vector unit, then does the same with the Value rows. It leaves one partial (reference maximum,
// sum of numerators, unnormalized output; log2 domain like the main kernel's partials) per (unit, head) in the
// partials array, where the main launch's split merge picks it up. It is launched before the main kernel on the
// same stream. The vector unit is enough here: the range is a small part of the context and its bytes are few.
#include "kvmix_common.hpp"

namespace kvmix {

namespace {

constexpr int kMixWaves = 8;
constexpr int kPitch = kD + 4;   // floats per staged row: rows of neighbouring tokens start 4 banks apart
constexpr int kHeads = 8;        // heads per workgroup at most

__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
// orders the wave's own LDS writes and reads (the staging area is wave-private)
__device__ __forceinline__ void wave_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ float h2f(uint32_t pair, int hh) { return (float)__builtin_bit_cast(half_t, (uint16_t)(pair >> (16 * hh))); }

// The 64 codes of 16-byte column l of a code section: (word j, half hh, slot) -> code.
template <int BITS> struct Column {
  uint32_t w[BITS == 4 ? 8 : 4];
  uint32_t h[2];
  __device__ __forceinline__ void load(const uint32_t* sec, int l) {
    if constexpr (BITS == 2 || BITS == 3 || BITS == 4) {
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(sec + 4 * l);
      w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
    }
    if constexpr (BITS == 4) {
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(sec + 256 + 4 * l);
      w[4] = v[0]; w[5] = v[1]; w[6] = v[2]; w[7] = v[3];
    }
    if constexpr (BITS == 1 || BITS == 3) {
      const u32x2_t v = *reinterpret_cast<const u32x2_t*>(sec + (BITS == 3 ? 256 : 0) + 2 * l);
      h[0] = v[0]; h[1] = v[1];
    }
  }
  __device__ __forceinline__ float code(int j, int hh, int slot) const {
    uint32_t c;
    if constexpr (BITS == 4) {
      c = (w[4 * (slot >> 2) + j] >> (16 * hh + 4 * (slot & 3))) & 15u;
    } else if constexpr (BITS == 1) {
      c = (h[j >> 1] >> (16 * hh + 8 * (j & 1) + 2 * (slot & 3) + (slot >> 2))) & 1u;
    } else {
      c = (w[j] >> (16 * hh + 2 * slot)) & 3u;
      if constexpr (BITS == 3) c += 4u * ((h[j >> 1] >> (16 * hh + 8 * (j & 1) + 2 * (slot & 3) + (slot >> 2))) & 1u);
    }
    return (float)c;
  }
};

// step of in-group element gi: the two 2-bit elements of a 3-bit group divide the same range by 3
template <int BITS> __device__ __forceinline__ float step_of(float s, bool two_bit_elem) {
  if (BITS == 3 && two_bit_elem) return (s * 7.0f) / 3.0f;
  return s;
}

template <int KB, int VB>
__global__ __launch_bounds__(kMixWaves * kWave) void mixed_fronts_kernel(MixedArgs a) {
  __shared__ __attribute__((aligned(16))) float X[kMixWaves][kTile][kPitch];   // one tile of Key rows, then of Value rows, as fp32;
                                                                               // at the end the wave's result [head][channel]
  __shared__ __attribute__((aligned(16))) float Q[kHeads][kD];
  __shared__ float P[kMixWaves][kHeads][kTile];   // softmax numerators of the tile
  __shared__ float Rm[kMixWaves][kHeads], Rl[kMixWaves][kHeads];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int u = blockIdx.x, uo = u * (int)gridDim.y + (int)blockIdx.y;   // (unit, head block): rows uo*G .. uo*G+G-1 of q
  const int G = a.G;
  for (int i = tid; i < G * kD; i += kMixWaves * kWave)
    Q[i / kD][i % kD] = (float)__builtin_bit_cast(half_t, a.q[(size_t)uo * G * kD + i]);
  __syncthreads();

  float m[kHeads], l[kHeads], o0[kHeads], o1[kHeads];   // running reference, sum, output channels lane and lane + 64
#pragma unroll
  for (int hh = 0; hh < kHeads; hh++) { m[hh] = -INFINITY; l[hh] = 0.0f; o0[hh] = 0.0f; o1[hh] = 0.0f; }

  float (&Xw)[kTile][kPitch] = X[wave];
  const int kq = lane >> 4, i16 = lane & 15;

  // ---- A tile's rows reach the staging area in two steps, request and conversion, so that the requests of the
  // next rows are in flight while the rows in hand are worked on.
  // fp16 ring rows: 16-byte piece lane + 64*jj is token (lane + 64*jj) / 16, channels 8*(lane % 16) .. +7.
  struct RingRaw { half8_t v[8]; };
  auto load_ring = [&](const uint16_t* ring, int t0, RingRaw& r) {
    // a row past the end is read from the last live token's slot instead (any slot is valid memory)
    const int s0 = (a.slot_begin + (t0 - a.t_begin)) % a.W_cap;
#pragma unroll
    for (int jj = 0; jj < 8; jj++) {
      const int tau = 4 * jj + kq;
      const int tc = t0 + tau < a.t_end ? tau : a.t_end - 1 - t0;
      int slot = s0 + tc;
      if (slot >= a.W_cap) slot -= a.W_cap;
      r.v[jj] = *reinterpret_cast<const half8_t*>(ring + ((size_t)u * a.W_cap + slot) * kD + 8 * i16);
    }
  };
  // rows of tokens from `first` on are written, rows at or past t_end as zeros
  auto conv_ring = [&](const RingRaw& r, int t0, int first) {
#pragma unroll
    for (int jj = 0; jj < 8; jj++) {
      const int tau = 4 * jj + kq, t = t0 + tau;
      const bool live = t < a.t_end;
      float4_t lo = float4_t{(float)r.v[jj][0], (float)r.v[jj][1], (float)r.v[jj][2], (float)r.v[jj][3]};
      float4_t hi = float4_t{(float)r.v[jj][4], (float)r.v[jj][5], (float)r.v[jj][6], (float)r.v[jj][7]};
      if (!live) { lo = float4_t{0, 0, 0, 0}; hi = lo; }
      if (t >= first) {
        *reinterpret_cast<float4_t*>(&Xw[tau][8 * i16]) = lo;
        *reinterpret_cast<float4_t*>(&Xw[tau][8 * i16 + 4]) = hi;
      }
    }
  };
  // a packed Key tile: lane = column l holds channels 32*ks + 8*kq + 2*j + hh of tokens 8*(i/4) + 4*m + i%4 (slot = ks + 4*m);
  // sm[4*ks + j] = (scale pair, minimum pair) of channels d, d + 1
  struct KeyRaw { Column<KB> col; u32x2_t sm[16]; };
  auto load_keys = [&](const uint32_t* rec, KeyRaw& r) {
    r.col.load(rec + kMetaWords, lane);
#pragma unroll
    for (int ks = 0; ks < 4; ks++)
#pragma unroll
      for (int j = 0; j < 4; j++) r.sm[4 * ks + j] = *reinterpret_cast<const u32x2_t*>(rec + 4 * (16 * ks + 4 * kq + j));
  };
  auto conv_keys = [&](const KeyRaw& r) {
    const int tau_m[2] = {8 * (i16 >> 2) + (i16 & 3), 8 * (i16 >> 2) + 4 + (i16 & 3)};
#pragma unroll
    for (int ks = 0; ks < 4; ks++)
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int hh = 0; hh < 2; hh++) {
          const float s = h2f(r.sm[4 * ks + j][0], hh), mn = h2f(r.sm[4 * ks + j][1], hh);
          const int d = 32 * ks + 8 * kq + 2 * j + hh;
#pragma unroll
          for (int mm = 0; mm < 2; mm++) {
            const int tau = tau_m[mm];
            const float prod = r.col.code(j, hh, ks + 4 * mm) * step_of<KB>(s, tau == 10 || tau == 21);
            Xw[tau][d] = prod + mn;
          }
        }
  };
  // a packed Value tile: lane = column l holds tokens 8*kq + 2*j + hh, channels 16*slot + i;
  // sm[4*g + j] = (scale pair, minimum pair) of the groups (tau, g), (tau + 1, g)
  struct ValueRaw { Column<VB> col; u32x2_t sm[16]; };
  auto load_values = [&](const uint32_t* rec, ValueRaw& r) {
    r.col.load(rec + kMetaWords + tile_words(KB), lane);
#pragma unroll
    for (int g = 0; g < 4; g++)
#pragma unroll
      for (int j = 0; j < 4; j++) r.sm[4 * g + j] = *reinterpret_cast<const u32x2_t*>(rec + 4 * (16 * g + 4 * kq + j) + 2);
  };
  auto conv_values = [&](const ValueRaw& r) {
#pragma unroll
    for (int g = 0; g < 4; g++)
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int hh = 0; hh < 2; hh++) {
          const float s = h2f(r.sm[4 * g + j][0], hh), mn = h2f(r.sm[4 * g + j][1], hh);
          const int tau = 8 * kq + 2 * j + hh;
#pragma unroll
          for (int sp = 0; sp < 2; sp++) {
            const int gi = 16 * sp + i16;
            const float prod = r.col.code(j, hh, 2 * g + sp) * step_of<VB>(s, gi == 10 || gi == 21);
            Xw[tau][32 * g + gi] = prod + mn;
          }
        }
  };
  // Where a tile's rows live (wave-uniform). Keys: packed before the Key front (a multiple of 32), else the ring.
  // Values: packed, ring, or - the tile in which the Value front stands - the record's rows up to the front and the
  // ring's from it on (what the record holds for those is unspecified).
  auto rec_of = [&](int t0) { return a.packed + ((size_t)u * a.tiles_cap + t0 / kTile) * (size_t)record_words(KB, VB); };
  auto keys_packed = [&](int t0) { return t0 < a.n_qk; };
  auto values_from_record = [&](int t0) { return t0 < a.n_qv; };
  auto values_from_ring = [&](int t0) { return t0 + kTile > a.n_qv; };
  RingRaw kr, vr;
  KeyRaw kp;
  ValueRaw vp;
  auto request_keys = [&](int t0) { if (keys_packed(t0)) load_keys(rec_of(t0), kp); else load_ring(a.k_win, t0, kr); };
  auto request_values = [&](int t0) {
    if (values_from_record(t0)) load_values(rec_of(t0), vp);
    if (values_from_ring(t0)) load_ring(a.v_win, t0, vr);
  };

  const int n_tiles = (a.t_end - a.t_begin + kTile - 1) / kTile;
  const int tau = lane & 31, part = lane >> 5;   // scores: lane (tau, part) sums channels 64*part .. 64*part + 63 of token tau
  if (wave < n_tiles) { request_keys(a.t_begin + wave * kTile); request_values(a.t_begin + wave * kTile); }
  for (int jt = wave; jt < n_tiles; jt += kMixWaves) {
    const int t0 = a.t_begin + jt * kTile, t_next = t0 + kMixWaves * kTile;
    const bool more = jt + kMixWaves < n_tiles;
    if (keys_packed(t0)) conv_keys(kp); else conv_ring(kr, t0, t0);
    if (more) request_keys(t_next);          // the Key registers are free again: the next tile's rows travel during the rest
    wave_fence();
    const bool live = t0 + tau < a.t_end;
    float s[kHeads];
#pragma unroll
    for (int hh = 0; hh < kHeads; hh++) s[hh] = 0.0f;
#pragma unroll 4
    for (int c = 0; c < 16; c++) {
      const float4_t x = *reinterpret_cast<const float4_t*>(&Xw[tau][64 * part + 4 * c]);
#pragma unroll
      for (int hh = 0; hh < kHeads; hh++) {
        if (hh < G) {
          const float4_t qv = *reinterpret_cast<const float4_t*>(&Q[hh][64 * part + 4 * c]);
          s[hh] += x[0] * qv[0] + x[1] * qv[1] + x[2] * qv[2] + x[3] * qv[3];
        }
      }
    }
#pragma unroll
    for (int hh = 0; hh < kHeads; hh++) {
      if (hh < G) {
        const float st = s[hh] + __shfl_xor(s[hh], 32);
        const float x = live ? st * a.scale_log2 : -INFINITY;
        const float mnew = fmaxf(m[hh], wave_max_f(x));     // finite: every tile has at least one live token
        const float f = exp2f(m[hh] - mnew);                // 0 on the wave's first tile
        const float p = exp2f(x - mnew);                    // 0 for rows past the end
        l[hh] = l[hh] * f + wave_sum_f(part == 0 ? p : 0.0f);
        o0[hh] *= f; o1[hh] *= f;
        m[hh] = mnew;
        if (part == 0) P[wave][hh][tau] = p;
      }
    }
    wave_fence();
    if (values_from_record(t0)) conv_values(vp);
    if (values_from_ring(t0)) {
      if (values_from_record(t0)) wave_fence();
      conv_ring(vr, t0, a.n_qv > t0 ? a.n_qv : t0);
    }
    if (more) request_values(t_next);
    wave_fence();
#pragma unroll 4
    for (int t = 0; t < kTile; t++) {
      const float x0 = Xw[t][lane], x1 = Xw[t][lane + kWave];
#pragma unroll
      for (int hh = 0; hh < kHeads; hh++) {
        if (hh < G) {
          const float p = P[wave][hh][t];
          o0[hh] += p * x0;
          o1[hh] += p * x1;
        }
      }
    }
    wave_fence();
  }

  // the wave's result into its own staging area (rows 0 .. G-1 hold [head][channel])
#pragma unroll
  for (int hh = 0; hh < kHeads; hh++) {
    if (hh < G) {
      if (lane == 0) { Rm[wave][hh] = m[hh]; Rl[wave][hh] = l[hh]; }
      Xw[hh][lane] = o0[hh];
      Xw[hh][lane + kWave] = o1[hh];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * kD; idx += kMixWaves * kWave) {
    const int hh = idx / kD, d = idx % kD;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kMixWaves; w++) M = fmaxf(M, Rm[w][hh]);
    float L = 0.0f, O = 0.0f;
#pragma unroll
    for (int w = 0; w < kMixWaves; w++) {
      const float f = Rm[w][hh] == -INFINITY ? 0.0f : exp2f(Rm[w][hh] - M);
      L += Rl[w][hh] * f;
      O += X[w][hh][d] * f;
    }
    float* pp = a.part + (((size_t)uo * a.n_parts + a.part_index) * G + hh) * (kD + 2);
    if (d == 0) { pp[0] = M; pp[1] = L; }
    pp[2 + d] = O;
  }
}

template <int KB, int VB>
hipError_t launch_mx(const MixedArgs& a, dim3 grid, hipStream_t s) {
  mixed_fronts_kernel<KB, VB><<<grid, kMixWaves * kWave, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_mixed_fronts(const MixedArgs& a, int units, int head_blocks, hipStream_t s) {
  if (units == 0 || a.t_end <= a.t_begin) return hipSuccess;
  const dim3 grid(units, head_blocks);
  switch (a.k_bits * 10 + a.v_bits) {
    case 11: return launch_mx<1, 1>(a, grid, s);
    case 12: return launch_mx<1, 2>(a, grid, s);
    case 13: return launch_mx<1, 3>(a, grid, s);
    case 14: return launch_mx<1, 4>(a, grid, s);
    case 21: return launch_mx<2, 1>(a, grid, s);
    case 31: return launch_mx<3, 1>(a, grid, s);
    case 41: return launch_mx<4, 1>(a, grid, s);
    case 22: return launch_mx<2, 2>(a, grid, s);
    case 23: return launch_mx<2, 3>(a, grid, s);
    case 24: return launch_mx<2, 4>(a, grid, s);
    case 32: return launch_mx<3, 2>(a, grid, s);
    case 33: return launch_mx<3, 3>(a, grid, s);
    case 34: return launch_mx<3, 4>(a, grid, s);
    case 42: return launch_mx<4, 2>(a, grid, s);
    case 43: return launch_mx<4, 3>(a, grid, s);
    case 44: return launch_mx<4, 4>(a, grid, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace kvmix
