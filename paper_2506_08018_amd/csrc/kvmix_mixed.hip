// Decode attention over the tokens that lie between the Key front and the Value front of a cache whose Keys and
// Values age separately (paper Sec. 3.3: the Recent Pivotal Context ratio of a layer's Keys and of its Values may
// differ; Sec. 3.2.2 step 4 for the dequantization).
//
// The main attention kernel works on tiles whose Keys and Values are both packed and on window tiles whose Keys and
// Values are both fp16. The tokens in between (a few tiles: at most the window's capacity) have one side packed and
// the other in the ring, and the Value front may stand inside a tile. This kernel takes them token by token, each
// Key row and each Value row from where it lives, in plain fp32 on the vector unit, and leaves one partial
// (reference maximum, sum of numerators, unnormalized output; log2 domain like the main kernel's partials) per
// (unit, head) in the partials array, where the main launch's split merge picks it up. It is launched before the
// main kernel on the same stream.
#include "kvmix_common.hpp"

namespace kvmix {

namespace {

constexpr int kMixWaves = 4;
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

__global__ __launch_bounds__(kMixWaves * kWave) void mixed_fronts_kernel(MixedArgs a) {
  __shared__ float X[kMixWaves][kTile][kPitch];   // one tile of Key rows, then of Value rows, as fp32
  __shared__ float Q[kHeads][kD];
  __shared__ float P[kMixWaves][kHeads][kTile];   // softmax numerators of the tile
  __shared__ float Rm[kMixWaves][kHeads], Rl[kMixWaves][kHeads];
  __shared__ float Ro[kMixWaves][kHeads][kD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int u = blockIdx.x, uo = u * (int)gridDim.y + (int)blockIdx.y;   // (unit, head block): rows uo*G .. uo*G+G-1 of q
  const int G = a.G;
  for (int i = tid; i < G * kD; i += kMixWaves * kWave)
    Q[i / kD][i % kD] = (float)__builtin_bit_cast(half_t, a.q[(size_t)uo * G * kD + i]);
  __syncthreads();

  float m[kHeads], l[kHeads], o0[kHeads], o1[kHeads];   // running reference, sum, output channels lane and lane + 64
#pragma unroll
  for (int hh = 0; hh < kHeads; hh++) { m[hh] = -INFINITY; l[hh] = 0.0f; o0[hh] = 0.0f; o1[hh] = 0.0f; }

  const size_t rec_words = (size_t)record_words(a.k_bits, a.v_bits);
  // one tile of rows into the staging area: which = 0 Keys, 1 Values; rows of tokens at or past t_end are zero
  auto stage = [&](int which, int t0) {
    const int front = which ? a.n_qv : a.n_qk;
    const uint16_t* ring = which ? a.v_win : a.k_win;
    for (int e = lane; e < kTile * kD; e += kWave) {
      const int tau = e / kD, d = e % kD, t = t0 + tau;
      float x = 0.0f;
      if (t < a.t_end) {
        if (t < front) {
          x = dequant_elem(a.packed + ((size_t)u * a.tiles_cap + t / kTile) * rec_words, a.k_bits, a.v_bits, which, tau, d);
        } else {
          const int slot = (a.slot_begin + (t - a.t_begin)) % a.W_cap;
          x = (float)__builtin_bit_cast(half_t, ring[((size_t)u * a.W_cap + slot) * kD + d]);
        }
      }
      X[wave][tau][d] = x;
    }
  };

  const int n_tiles = (a.t_end - a.t_begin + kTile - 1) / kTile;
  const int tau = lane & 31, part = lane >> 5;   // scores: lane (tau, part) sums channels 64*part .. 64*part + 63 of token tau
  for (int jt = wave; jt < n_tiles; jt += kMixWaves) {
    const int t0 = a.t_begin + jt * kTile;
    stage(0, t0);
    wave_fence();
    const bool live = t0 + tau < a.t_end;
#pragma unroll
    for (int hh = 0; hh < kHeads; hh++) {
      if (hh < G) {
        float s = 0.0f;
        for (int d = 0; d < kD / 2; d++) s += Q[hh][64 * part + d] * X[wave][tau][64 * part + d];
        s += __shfl_xor(s, 32);
        const float x = live ? s * a.scale_log2 : -INFINITY;
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
    stage(1, t0);
    wave_fence();
#pragma unroll
    for (int hh = 0; hh < kHeads; hh++) {
      if (hh < G) {
        float a0 = o0[hh], a1 = o1[hh];
        for (int t = 0; t < kTile; t++) {
          const float p = P[wave][hh][t];
          a0 += p * X[wave][t][lane];
          a1 += p * X[wave][t][lane + kWave];
        }
        o0[hh] = a0; o1[hh] = a1;
      }
    }
    wave_fence();
  }

#pragma unroll
  for (int hh = 0; hh < kHeads; hh++) {
    if (hh < G) {
      if (lane == 0) { Rm[wave][hh] = m[hh]; Rl[wave][hh] = l[hh]; }
      Ro[wave][hh][lane] = o0[hh];
      Ro[wave][hh][lane + kWave] = o1[hh];
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
      O += Ro[w][hh][d] * f;
    }
    float* pp = a.part + (((size_t)uo * a.n_parts + a.part_index) * G + hh) * (kD + 2);
    if (d == 0) { pp[0] = M; pp[1] = L; }
    pp[2 + d] = O;
  }
}

}  // namespace

hipError_t launch_mixed_fronts(const MixedArgs& a, int units, int head_blocks, hipStream_t s) {
  if (units == 0 || a.t_end <= a.t_begin) return hipSuccess;
  mixed_fronts_kernel<<<dim3(units, head_blocks), kMixWaves * kWave, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace kvmix
