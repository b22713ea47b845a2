// Decode attention over the tokens that lie between the Key front and the Value front of a cache whose Keys and
// Values age separately (paper Sec. 3.3: the Recent Pivotal Context ratio of a layer's Keys and of its Values may
// differ; Sec. 3.2.2 step 4 for the dequantization).
//
// The main attention kernel works on tiles whose Keys and Values are both packed and on window tiles whose Keys and
// Values are both fp16. The tokens in between ((r_k - r_v) x context of them under the count formula) have one
// side packed and the other in the ring, and the Value front may stand inside a tile. This kernel takes them, tile
// by tile and a wave per tile, in registers on the vector unit:
//   - a packed side is unpacked by the lane that loaded it (the 64 codes of its 16-byte column, x = code * s_i + min),
//     a ring side is read as 16-byte row pieces (lane = tokens 8*(lane/16) + jj, channels 8*(lane%16) .. +7);
//   - scores are per-lane partial dot products reduced across the lanes that share a token; numerators are kept
//     per token row (tokens 8*(lane/16) .. +7), which is the token ownership of both Value forms;
//   - a lane accumulates the output channels it holds Values for (8 per lane: 16*slot + lane%16 from a record,
//     8*(lane%16) .. +7 from the ring) over its row's tokens; the rows are added up once at the end;
//   - the tile in which the Value front stands is worked on twice, by a wave in each Value form, each with the
//     numerators of the other's tokens set to zero, so a wave's accumulators keep one channel ownership.
// It leaves one partial (reference maximum, sum of numerators, unnormalized output; log2 domain like the main
// kernel's partials) per (unit, head) in the partials array, where the main launch's split merge picks it up. It is
// launched before the main kernel on the same stream. The vector unit is enough here: the range is a side path.
#include <type_traits>
#include "kvmix_common.hpp"

namespace kvmix {

namespace {

constexpr int kMixWaves = 8;

typedef float float2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float xor16(float v) { return __shfl_xor(v, 16); }
__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
// sum over the 16 lanes of each row (lanes that share lane/16); every lane of the row gets it
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);   // row_half_mirror
  v += dpp_f<0x140>(v);   // row_mirror
  return v;
}
// orders the wave's own LDS writes and reads
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

// step of an in-group element: the two 2-bit elements of a 3-bit group divide the same range by 3
template <int BITS> __device__ __forceinline__ float step_of(float s, bool two_bit_elem) {
  if (BITS == 3 && two_bit_elem) return (s * 7.0f) / 3.0f;
  return s;
}

// GH: query heads per workgroup (1, 2 or 4). V_AHEAD: the Value front is ahead of the Key front, i.e. in the whole
// range the Keys come from the ring and the Values from the records (but for the tokens from the Value front on);
// otherwise the Keys come from the records and the Values from the ring (but for the tokens before the Value front).
template <int KB, int VB, int GH, bool V_AHEAD>
__global__ __launch_bounds__(kMixWaves * kWave) void mixed_fronts_kernel(MixedArgs a) {
  __shared__ float O[kMixWaves][GH][kD];          // per-wave results
  __shared__ float Rm[kMixWaves][GH], Rl[kMixWaves][GH];
  __shared__ __attribute__((aligned(16))) float P[kMixWaves][GH][kTile];   // Keys from records: scores by token
  __shared__ __attribute__((aligned(16))) float Q[GH][kD];                 // Keys from records: the query as fp32

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kq = lane >> 4, i16 = lane & 15;
  const int u = blockIdx.x, head0 = (int)blockIdx.y * GH;     // first query head of this workgroup within the unit's group
  const uint16_t* qg = a.q + ((size_t)u * a.G + head0) * kD;

  // the query: Keys from the ring meet it as fp16 pairs in the row form (channels 8*i16 .. +7), Keys from records
  // as fp32 at the channels a column holds
  half2_t qh[GH][4];
  if constexpr (V_AHEAD) {
#pragma unroll
    for (int hh = 0; hh < GH; hh++) {
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(qg + hh * kD + 8 * i16);
#pragma unroll
      for (int c = 0; c < 4; c++) {
        const uint32_t w = v[c];      // a copy: a bit cast applied to the vector element itself reads element 0
        qh[hh][c] = __builtin_bit_cast(half2_t, w);
      }
    }
  } else {
    for (int i = tid; i < GH * kD; i += kMixWaves * kWave) Q[i / kD][i % kD] = (float)__builtin_bit_cast(half_t, qg[i]);
    __syncthreads();
  }

  float m[GH], l[GH], o[GH][8];      // running reference (wave-uniform), sum of the row's numerators, the lane's 8 channels
#pragma unroll
  for (int hh = 0; hh < GH; hh++) {
    m[hh] = -INFINITY; l[hh] = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; c++) o[hh][c] = 0.0f;
  }

  // Work items. The main items are the range's tiles in the Value form that most of the range has (records when the
  // Value front is ahead, the ring otherwise), shared by waves 0 .. n_main_waves-1; the tokens on the other side of
  // the Value front inside its tile are one more item, in the other Value form, for the last wave.
  const int n_tiles = (a.t_end - a.t_begin + kTile - 1) / kTile;
  const bool split_tile = V_AHEAD ? a.n_qv < a.t_end : a.n_qv > a.t_begin;
  const int n_main_waves = split_tile ? kMixWaves - 1 : kMixWaves;
  const bool special = split_tile && wave == kMixWaves - 1;
  const bool values_packed = V_AHEAD != special;               // the Value form of this wave's items
  // token range whose numerators count for this wave (the rest belongs to the other form's item)
  const int tok_lo = values_packed ? a.t_begin : (a.n_qv > a.t_begin ? a.n_qv : a.t_begin);
  const int tok_hi = values_packed ? (a.n_qv < a.t_end ? a.n_qv : a.t_end) : a.t_end;
  int jt = special ? (V_AHEAD ? n_tiles - 1 : 0) : wave;
  const int jt_step = special ? n_tiles : n_main_waves;
  const size_t rec_words = (size_t)record_words(KB, VB);

  // The whole tile loop exists once per Value form (the form is a compile-time constant inside): a wave runs one of
  // the two, and the registers of the other form's rows are never allocated next to its own.
  auto run = [&](auto vform) {
  constexpr bool VP = decltype(vform)::value;        // Values from the records
  // What a tile needs from memory, as requested. (Requesting the next tile's set as well before working on this one
  // measured slower: twice the requests at the start of the launch delay every wave's first tile.)
  struct Raw {
    half8_t kr[V_AHEAD ? 8 : 1];                                  // Keys from the ring: row pieces
    Column<KB> kcol; u32x2_t ksm[V_AHEAD ? 1 : 16];               // Keys from a record: the lane's column, (scale pair, minimum pair) of its channels
    half8_t vr[VP ? 1 : 8];                                       // Values from the ring
    Column<VB> vcol; u32x2_t vsm[VP ? 16 : 1];                    // Values from a record
  };
  auto request = [&](Raw& r, int tile) {
    const int t0 = a.t_begin + tile * kTile;
    const uint32_t* rec = a.packed + ((size_t)u * a.tiles_cap + t0 / kTile) * rec_words;
    const int s0 = (a.slot_begin + (t0 - a.t_begin)) % a.W_cap;          // ring slot of the tile's first token
    // ring row piece of token 8*kq + jj of the tile if it lies inside [lo, hi), else of the nearest token inside:
    // every slot read holds a live token, and what is read for a token outside only ever meets a zero numerator
    auto row_ptr = [&](const uint16_t* ring, int jj, int lo, int hi) {
      int t = t0 + 8 * kq + jj;
      t = t < lo ? lo : t;
      t = t >= hi ? hi - 1 : t;
      int slot = s0 + (t - t0);
      if (slot < 0) slot += a.W_cap;
      if (slot >= a.W_cap) slot -= a.W_cap;
      return ring + ((size_t)u * a.W_cap + slot) * kD + 8 * i16;
    };
    if constexpr (V_AHEAD) {
#pragma unroll
      for (int jj = 0; jj < 8; jj++) r.kr[jj] = *reinterpret_cast<const half8_t*>(row_ptr(a.k_win, jj, a.t_begin, a.t_end));
    } else {
      r.kcol.load(rec + kMetaWords, lane);
#pragma unroll
      for (int ks = 0; ks < 4; ks++)
#pragma unroll
        for (int j = 0; j < 4; j++) r.ksm[4 * ks + j] = *reinterpret_cast<const u32x2_t*>(rec + 4 * (16 * ks + 4 * kq + j));
    }
    if constexpr (VP) {
      r.vcol.load(rec + kMetaWords + tile_words(KB), lane);
#pragma unroll
      for (int g = 0; g < 4; g++)
#pragma unroll
        for (int j = 0; j < 4; j++) r.vsm[4 * g + j] = *reinterpret_cast<const u32x2_t*>(rec + 4 * (16 * g + 4 * kq + j) + 2);
    } else {
#pragma unroll
      for (int jj = 0; jj < 8; jj++) r.vr[jj] = *reinterpret_cast<const half8_t*>(row_ptr(a.v_win, jj, tok_lo, tok_hi));
    }
  };
  Raw cur;
  for (; jt < n_tiles; jt += jt_step) {
    const int t0 = a.t_begin + jt * kTile;
    request(cur, jt);
    // all requests are issued here: nothing is scheduled across this point (left to itself the compiler moves each
    // load down to its first use, and the uses then wait for their loads one by one)
    __builtin_amdgcn_sched_barrier(0);
    const auto& kr = cur.kr; const auto& kcol = cur.kcol; const auto& ksm = cur.ksm;
    const auto& vr = cur.vr; const auto& vcol = cur.vcol; const auto& vsm = cur.vsm;

    // ---- scores of the tokens 8*kq + jj (log2 domain), the same in all 16 lanes of a row
    float p[GH][8];
    if constexpr (V_AHEAD) {
      // lane: 8 channels of 8 tokens; packed dot products, then the sum over the 16 lanes of the row
#pragma unroll
      for (int hh = 0; hh < GH; hh++)
#pragma unroll
        for (int jj = 0; jj < 8; jj++) {
          const u32x4_t r = __builtin_bit_cast(u32x4_t, kr[jj]);
          float s = 0.0f;
#pragma unroll
          for (int c = 0; c < 4; c++) {
            const uint32_t w = r[c];    // (a copy, as above)
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w), qh[hh][c], s, false);
          }
          p[hh][jj] = row_sum(s) * a.scale_log2;
        }
    } else {
      // lane = column l: channels 32*ks + 8*kq + 2*j + hc of tokens tau_m = 8*(i16/4) + 4*m + i16%4 (slot = ks + 4*m);
      // partial sums over the lane's 32 channels, summed over the four kq, then handed to the token rows through LDS
      float sc[GH][2];
#pragma unroll
      for (int hh = 0; hh < GH; hh++) { sc[hh][0] = 0.0f; sc[hh][1] = 0.0f; }
      const int tau_m[2] = {8 * (i16 >> 2) + (i16 & 3), 8 * (i16 >> 2) + 4 + (i16 & 3)};
#pragma unroll
      for (int ks = 0; ks < 4; ks++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          float x[2][2];       // [channel of the pair][token]
#pragma unroll
          for (int hc = 0; hc < 2; hc++) {
            const float s = h2f(ksm[4 * ks + j][0], hc), mn = h2f(ksm[4 * ks + j][1], hc);
#pragma unroll
            for (int mm = 0; mm < 2; mm++) {
              const float prod = kcol.code(j, hc, ks + 4 * mm) * step_of<KB>(s, tau_m[mm] == 10 || tau_m[mm] == 21);
              x[hc][mm] = prod + mn;
            }
          }
#pragma unroll
          for (int hh = 0; hh < GH; hh++) {
            const float2_t q2 = *reinterpret_cast<const float2_t*>(&Q[hh][32 * ks + 8 * kq + 2 * j]);
#pragma unroll
            for (int mm = 0; mm < 2; mm++) sc[hh][mm] += q2[0] * x[0][mm] + q2[1] * x[1][mm];
          }
          // keeps the query reads of the following channel pairs behind this pair's arithmetic: hoisted together
          // (64 of them at 4 heads) they do not fit the register file
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
      for (int hh = 0; hh < GH; hh++)
#pragma unroll
        for (int mm = 0; mm < 2; mm++) {
          float s = sc[hh][mm];
          s += xor16(s);
          s += xor32(s);
          if (kq == 0) P[wave][hh][tau_m[mm]] = s * a.scale_log2;
        }
      wave_fence();
#pragma unroll
      for (int hh = 0; hh < GH; hh++) {
        const float4_t lo = *reinterpret_cast<const float4_t*>(&P[wave][hh][8 * kq]);
        const float4_t hi = *reinterpret_cast<const float4_t*>(&P[wave][hh][8 * kq + 4]);
#pragma unroll
        for (int c = 0; c < 4; c++) { p[hh][c] = lo[c]; p[hh][4 + c] = hi[c]; }
      }
      wave_fence();     // the next tile's scores are written after these reads
    }

    // ---- online softmax per head over the wave's tokens; numerators of tokens outside [tok_lo, tok_hi) are zero
#pragma unroll
    for (int hh = 0; hh < GH; hh++) {
      float mx = -INFINITY;
#pragma unroll
      for (int jj = 0; jj < 8; jj++) {
        const int t = t0 + 8 * kq + jj;
        p[hh][jj] = (t >= tok_lo && t < tok_hi) ? p[hh][jj] : -INFINITY;
        mx = fmaxf(mx, p[hh][jj]);
      }
      mx = fmaxf(mx, xor16(mx));
      mx = fmaxf(mx, xor32(mx));
      const float mnew = fmaxf(m[hh], mx);
      const bool none = mnew == -INFINITY;          // no token of this wave's range so far (wave-uniform)
      const float f = none ? 1.0f : exp2f(m[hh] - mnew);        // 0 on the first tile with tokens
      float ps = 0.0f;
#pragma unroll
      for (int jj = 0; jj < 8; jj++) {
        p[hh][jj] = none ? 0.0f : exp2f(p[hh][jj] - mnew);      // 0 for tokens outside the range
        ps += p[hh][jj];
      }
      l[hh] = l[hh] * f + ps;
      m[hh] = mnew;
#pragma unroll
      for (int c = 0; c < 8; c++) o[hh][c] *= f;
    }

    // ---- Values: the lane's 8 channels over its row's 8 tokens
    if constexpr (VP) {
      // lane = column l: tokens 8*kq + 2*j + hc (jj = 2*j + hc), channels 16*slot + i16: o[.][slot]
#pragma unroll
      for (int g = 0; g < 4; g++)
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
          for (int hc = 0; hc < 2; hc++) {
            const int jj = 2 * j + hc;
            // a token at or past the Value front has nothing defined in the record: its scale and minimum count as 0
            const bool defined = t0 + 8 * kq + jj < a.n_qv;
            const float s = defined ? h2f(vsm[4 * g + j][0], hc) : 0.0f, mn = defined ? h2f(vsm[4 * g + j][1], hc) : 0.0f;
#pragma unroll
            for (int sp = 0; sp < 2; sp++) {
              const int gi = 16 * sp + i16;
              const float prod = vcol.code(j, hc, 2 * g + sp) * step_of<VB>(s, gi == 10 || gi == 21);
              const float x = prod + mn;
#pragma unroll
              for (int hh = 0; hh < GH; hh++) o[hh][2 * g + sp] += p[hh][jj] * x;
            }
          }
    } else {
      // lane: channels 8*i16 + c of tokens 8*kq + jj: o[.][c]
#pragma unroll
      for (int jj = 0; jj < 8; jj++)
#pragma unroll
        for (int c = 0; c < 8; c++) {
          const float x = (float)vr[jj][c];
#pragma unroll
          for (int hh = 0; hh < GH; hh++) o[hh][c] += p[hh][jj] * x;
        }
    }
  }

  // ---- the wave's result: rows added up, channels to their places
#pragma unroll
  for (int hh = 0; hh < GH; hh++) {
    float lt = l[hh];
    lt += xor16(lt);
    lt += xor32(lt);
#pragma unroll
    for (int c = 0; c < 8; c++) {
      float v = o[hh][c];
      v += xor16(v);
      v += xor32(v);
      if (kq == 0) O[wave][hh][VP ? 16 * c + i16 : 8 * i16 + c] = v;
    }
    if (lane == 0) { Rm[wave][hh] = m[hh]; Rl[wave][hh] = lt; }
  }
  };
  if (values_packed) run(std::true_type{}); else run(std::false_type{});
  __syncthreads();
  // the partial of head hg (within the unit's group) goes where the main kernel's merge looks for it: that kernel
  // numbers (unit, block of G_main heads) pairs
  for (int idx = tid; idx < GH * kD; idx += kMixWaves * kWave) {
    const int hh = idx / kD, d = idx % kD;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kMixWaves; w++) M = fmaxf(M, Rm[w][hh]);
    float L = 0.0f, Ov = 0.0f;
#pragma unroll
    for (int w = 0; w < kMixWaves; w++) {
      const bool has = Rm[w][hh] != -INFINITY;
      const float f = has ? exp2f(Rm[w][hh] - M) : 0.0f;
      L += Rl[w][hh] * f;
      Ov += (has ? O[w][hh][d] : 0.0f) * f;
    }
    const int hg = head0 + hh;
    const int blocks = a.G / a.G_main;
    const size_t uo = (size_t)u * blocks + hg / a.G_main;
    float* pp = a.part + ((uo * a.n_parts + a.part_index) * a.G_main + hg % a.G_main) * (kD + 2);
    if (d == 0) { pp[0] = M; pp[1] = L; }
    pp[2 + d] = Ov;
  }
}

template <int KB, int VB, int GH, bool V_AHEAD>
hipError_t launch_mx(const MixedArgs& a, int units, hipStream_t s) {
  mixed_fronts_kernel<KB, VB, GH, V_AHEAD><<<dim3(units, a.G / GH), kMixWaves * kWave, 0, s>>>(a);
  return hipGetLastError();
}

// Heads per workgroup: up to 4 when the Keys come from the ring. With Keys from the records one head per workgroup:
// unpacking a Key column against several heads at once (the query values of 32 channels per head and lane) does not
// fit the register file, and a spilling kernel is slower than the repeated unpacking.
template <int KB, int VB>
hipError_t launch_gh(const MixedArgs& a, int units, hipStream_t s) {
  if (a.n_qv <= a.n_qk) return launch_mx<KB, VB, 1, false>(a, units, s);
  switch (a.G >= 4 ? 4 : a.G) {
    case 1: return launch_mx<KB, VB, 1, true>(a, units, s);
    case 2: return launch_mx<KB, VB, 2, true>(a, units, s);
    case 4: return launch_mx<KB, VB, 4, true>(a, units, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_mixed_fronts(const MixedArgs& a, int units, hipStream_t s) {
  if (units == 0 || a.t_end <= a.t_begin) return hipSuccess;
  switch (a.k_bits * 10 + a.v_bits) {
    case 11: return launch_gh<1, 1>(a, units, s);
    case 12: return launch_gh<1, 2>(a, units, s);
    case 13: return launch_gh<1, 3>(a, units, s);
    case 14: return launch_gh<1, 4>(a, units, s);
    case 21: return launch_gh<2, 1>(a, units, s);
    case 31: return launch_gh<3, 1>(a, units, s);
    case 41: return launch_gh<4, 1>(a, units, s);
    case 22: return launch_gh<2, 2>(a, units, s);
    case 23: return launch_gh<2, 3>(a, units, s);
    case 24: return launch_gh<2, 4>(a, units, s);
    case 32: return launch_gh<3, 2>(a, units, s);
    case 33: return launch_gh<3, 3>(a, units, s);
    case 34: return launch_gh<3, 4>(a, units, s);
    case 42: return launch_gh<4, 2>(a, units, s);
    case 43: return launch_gh<4, 3>(a, units, s);
    case 44: return launch_gh<4, 4>(a, units, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace kvmix
