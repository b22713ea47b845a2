// Fused decode attention over the packed mixed-bit KV cache plus the fp16 recent window (gfx950).
//
// Paper Sec. 3.4 item 2 (dequantize on the fly while multiplying, never materialize fp16 K/V),
// Sec. 3.2.2 step 4 (x = q*s + min), Sec. 3.3 (recent tokens stay in full precision).
//
// Formulation. For one kv head and one 32-token tile
//   score[t][h] = sum_d code[t][d] * (q[h][d]*s[d])  +  sum_d q[h][d]*z[d]
//   out[d][h]  += sum_t code[t][d] * (p[t][h]*s[t][g(d)])  +  sum_t p[t][h]*z[t][g(d)]
// Both code sums are 16x16x32 fp16 MFMAs whose A operand is the packed word ANDed with a mask:
// a 1/2/4-bit field left in place inside a zero fp16 pattern is the subnormal code * 2^(pos-24),
// exact, and MFMA honours subnormal inputs (3-bit codes are a 2-bit plane plus a 1-bit plane). The scale factors ride in the B operand, split
// into an fp16 (hi, lo) pair held in two MFMA columns so that the products stay exact to
// ~22 bits; the up-to-8 query heads of the group use columns 0..7 (hi) and 8..15 (lo).
// The fp16 window runs on MFMAs with plain fp16 operands; so do the zero-point sums for groups of
// 4 or 8 query heads, while groups of 1 or 2 heads take them (and the softmax denominator) on the
// vector unit, where they are cheaper than matrix instructions with mostly empty columns.
//
// Data movement. Every byte of a tile record is loaded from HBM once, by one lane (16 B of
// metadata and 16 B of every 1 KiB of codes per lane); a wave has one tile in flight while the
// other waves of its SIMD compute. The scale-folded
// B operands are computed cooperatively (each lane two values per head) and redistributed
// through a wave-private LDS area, so no barrier is needed inside the main loop.
// Softmax is online, per wave, with a lazily raised reference maximum; waves of a workgroup
// take tiles from a shared counter and merge through LDS (without a barrier when the unit is not
// split: the last wave to deliver combines); splits of one unit merge through a workspace, the
// last arriving workgroup writes the output.
#include "kvmix_common.hpp"

namespace kvmix {

namespace {

// waves per workgroup: 3 per SIMD where the LDS exchange areas fit (register budget 512 / 3 per lane)
constexpr int waves_for(int G) { return 12; }
constexpr int kDepth = 1;            // tiles a wave requests ahead; 2 and 3 measured no faster (the loop runs at the memory system's rate)
constexpr int kMergeBatch = 32;          // splits whose partials the merging workgroup requests together (one round trip)
// Reference of the running softmax (log2 units): numerators 2^(score - reference) are kept at or below 2^kRefCap;
// when a score would exceed that, the reference is raised to (that score - kRefCap + 4), which leaves room for
// scores 16 times larger before the next raise. Numerators are large on purpose: they and their products with
// the Value scales travel as fp16 pairs whose absolute resolution is 2^-25, and the thousands of low-weight
// tokens of a long context sit near that floor; with numerators up to 2^6 instead of 1 the floor is 64 times
// lower relative to the sums. The price is the range: a Value group scale must stay below 2^16 / 2^6 = 1024.
constexpr float kRefCap = 6.0f;
constexpr float kRefMargin = 4.0f - kRefCap;

typedef float float2_t __attribute__((ext_vector_type(2)));

// 2^x by the hardware instruction alone (results below 2^-126 flush to zero, which is harmless here)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float4_t mfma16(half8_t a, half8_t b, float4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
// value of lane (l ^ 8) within each row of 16 lanes
__device__ __forceinline__ float ror8(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false));
}
__device__ __forceinline__ half8_t as_half8(u32x4_t v) { return __builtin_bit_cast(half8_t, v); }
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_f(float v) {   // lanes without a source (or outside ROW_MASK) read 0
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}
// sum over the 16 lanes of each row; every lane of the row gets it
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);   // row_half_mirror
  v += dpp_f<0x140>(v);   // row_mirror
  return v;
}
// maximum over the 16 lanes of each row; every lane of the row gets it
__device__ __forceinline__ float row_max(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  v = fmaxf(v, dpp_f<0x141>(v));
  v = fmaxf(v, dpp_f<0x140>(v));
  return v;
}
// sum over the 64 lanes of the wave as a wave-uniform value
__device__ __forceinline__ float wave_sum(float v) {
  v = row_sum(v);
  v += dpp_f<0x142, 0xA>(v);   // row_bcast:15 -> rows 1 and 3 add the sum of the row before
  v += dpp_f<0x143, 0xC>(v);   // row_bcast:31 -> rows 2 and 3 add the sum of rows 0..1
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {   // rare path: plain butterflies
  v = fmaxf(v, __shfl_xor(v, 1)); v = fmaxf(v, __shfl_xor(v, 2)); v = fmaxf(v, __shfl_xor(v, 4));
  v = fmaxf(v, __shfl_xor(v, 8)); v = fmaxf(v, __shfl_xor(v, 16)); v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ __forceinline__ float uniform_lane(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
// orders the wave's own LDS writes before its following LDS reads (LDS executes a wave's
// operations in order; this only pins the compiler)
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Bit position (inside a 16-bit half, after the unpack shift) of the field that feeds slot `s`
// (0..3 = slot % 4): the MFMA sees code * 2^(pos - 24). Fields are moved as high in the fp16 mantissa
// as they fit: the matrix core aligns the products of one dot product to their largest nominal
// exponent (that of a subnormal is fixed) and truncates below its window, so a code sitting in the
// lowest mantissa bits loses product bits (measured: ~1e-5 relative at position 0, exact from 6 up).
template <int BITS> __device__ __forceinline__ constexpr int field_pos(int s) { return BITS == 4 ? 4 * (s & 1) + 2 : BITS == 1 ? 2 * s + 4 : 2 * s + 2; }

// ---- A operands from packed words. wa = word << 2, wb = word >> 6 (slots 0..3 / 4..7 of each half).
// 2-bit plane (also the low plane of 3-bit): slot field from bits 2*slot to bits 2*(slot%4) + 2.
__device__ __forceinline__ half8_t unpack2(const u32x4_t& wa, const u32x4_t& wb, int slot) {
  const uint32_t mask = 0x00030003u << (2 * (slot & 3) + 2);
  const u32x4_t src = (slot & 4) ? wb : wa;
  return as_half8(src & mask);
}
// 4-bit: 8 words (two chunks of 4), slot -> chunk slot/4, field slot%4 from bits 4*field to 4*(field%2) + 2.
__device__ __forceinline__ half8_t unpack4(const u32x4_t& wa, const u32x4_t& wb, int field) {
  const uint32_t mask = 0x000F000Fu << (4 * (field & 1) + 2);
  const u32x4_t src = (field & 2) ? wb : wa;
  return as_half8(src & mask);
}
// 1-bit high plane of 3-bit codes: 2 words; word j/2 holds, for pair j, bit 8*(j%2) + 2*(slot%4) + slot/4.
// hs[v] = plane shifted so that variant v = 2*(j%2) + slot/4 has its bits at 2*(slot%4) + 4, two above
// the low plane's field (bit 10, the lowest exponent bit, continues the subnormal scale: 2^-14).
__device__ __forceinline__ half8_t unpack1(const u32x2_t (&hs)[4], int slot) {
  const uint32_t mask = 0x00010001u << (2 * (slot & 3) + 4);
  const int hi = slot >> 2;
  u32x4_t r;
  r[0] = hs[0 + hi][0] & mask;   // j = 0: word 0, variant (0, hi)
  r[1] = hs[2 + hi][0] & mask;   // j = 1: word 0, variant (1, hi)
  r[2] = hs[0 + hi][1] & mask;   // j = 2: word 1
  r[3] = hs[2 + hi][1] & mask;   // j = 3: word 1
  return as_half8(r);
}
__device__ __forceinline__ void shift_hi_plane(const u32x2_t& h, u32x2_t (&hs)[4]) {
  hs[0] = h << 4;   // (j%2 = 0, slot/4 = 0): source bit 2*s     -> 2*s + 4
  hs[1] = h << 3;   // (0, 1):                 source bit 2*s + 1 -> 2*s + 4
  hs[2] = h >> 4;   // (1, 0):                 source bit 2*s + 8 -> 2*s + 4
  hs[3] = h >> 5;   // (1, 1):                 source bit 2*s + 9 -> 2*s + 4
}

// Tile loads are buffer loads: a unit's array is one buffer resource (scalar registers), the tile's
// byte offset a scalar operand and the lane's offset one 32-bit vector register, so a load costs no
// address arithmetic. Reads beyond the resource's size return zero instead of faulting.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  // the base is wave-uniform by construction; saying so keeps the descriptor in scalar registers
  const uint64_t v = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  void* ub = reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(ub, 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
// Cache policy of the tile loads: non-temporal. Every record is read once per launch; marked as streaming it
// does not displace other lines on its way through the caches (measured: 1.5 us less per launch on the
// Llama-2-7B-shaped workload).
constexpr int kStreaming = 2;
__device__ __forceinline__ u32x4_t buf_load16(rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, kStreaming));
}
__device__ __forceinline__ u32x2_t buf_load8(rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(u32x2_t, __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, kStreaming));
}

// The lane's share of one packed tile as loaded (Raw) and prepared for unpacking (Codes).
template <int BITS> struct Raw;
template <> struct Raw<1> {     // the bit plane alone: 8 bytes per lane
  u32x2_t h;
  __device__ __forceinline__ void load(rsrc_t r, uint32_t soff, uint32_t, uint32_t l8) { h = buf_load8(r, l8, soff); }
};
template <> struct Raw<2> {
  u32x4_t w;
  __device__ __forceinline__ void load(rsrc_t r, uint32_t soff, uint32_t l16, uint32_t) { w = buf_load16(r, l16, soff); }
};
template <> struct Raw<3> {
  u32x4_t w; u32x2_t h;
  __device__ __forceinline__ void load(rsrc_t r, uint32_t soff, uint32_t l16, uint32_t l8) {
    w = buf_load16(r, l16, soff);
    h = buf_load8(r, l8, soff + 1024u);
  }
};
template <> struct Raw<4> {
  u32x4_t w[2];
  __device__ __forceinline__ void load(rsrc_t r, uint32_t soff, uint32_t l16, uint32_t) {
    w[0] = buf_load16(r, l16, soff);
    w[1] = buf_load16(r, l16, soff + 1024u);
  }
};
template <int BITS> struct Codes;
template <> struct Codes<1> {
  u32x2_t hs[4];
  __device__ __forceinline__ explicit Codes(const Raw<1>& r) { shift_hi_plane(r.h, hs); }
  __device__ __forceinline__ half8_t lo(int slot) const { return unpack1(hs, slot); }
};
template <> struct Codes<2> {
  u32x4_t wa, wb;
  __device__ __forceinline__ explicit Codes(const Raw<2>& r) : wa(r.w << 2), wb(r.w >> 6) {}
  __device__ __forceinline__ half8_t lo(int slot) const { return unpack2(wa, wb, slot); }
};
template <> struct Codes<3> {
  u32x4_t wa, wb; u32x2_t hs[4];
  __device__ __forceinline__ explicit Codes(const Raw<3>& r) : wa(r.w << 2), wb(r.w >> 6) { shift_hi_plane(r.h, hs); }
  // the 2-bit field with the plane's bit right above it: one 3-bit field, the subnormal (or, with the bit at
  // position 10, smallest normal) fp16 number code * 2^(pos - 24)
  __device__ __forceinline__ half8_t lo(int slot) const {
    return as_half8(__builtin_bit_cast(u32x4_t, unpack2(wa, wb, slot)) | __builtin_bit_cast(u32x4_t, unpack1(hs, slot)));
  }
};
template <> struct Codes<4> {
  u32x4_t wa[2], wb[2];
  __device__ __forceinline__ explicit Codes(const Raw<4>& r) { wa[0] = r.w[0] << 2; wa[1] = r.w[1] << 2; wb[0] = r.w[0] >> 6; wb[1] = r.w[1] >> 6; }
  __device__ __forceinline__ half8_t lo(int slot) const { return unpack4(wa[slot >> 2], wb[slot >> 2], slot & 3); }
};

// One tile in flight: the lane's 16 bytes of metadata (Key scale pair, Key minimum pair, Value scale
// pair, Value minimum pair) and its share of the two code sections. The record of a tile is contiguous
// in memory, so a tile is three to five full-width loads from one stream.
template <int KB, int VB> struct Stage {
  u32x4_t meta;
  Raw<KB> kc; Raw<VB> vc;
  // rec: buffer resource over the unit's records; t: tile index inside the unit (wave-uniform)
  __device__ __forceinline__ void load(rsrc_t rec, int t, int lane) {
    const uint32_t l16 = 16u * lane, l8 = 8u * lane;
    const uint32_t soff = (uint32_t)t * (uint32_t)(record_words(KB, VB) * 4);
    meta = buf_load16(rec, l16, soff);
    kc.load(rec, soff + (uint32_t)(kMetaWords * 4), l16, l8);
    vc.load(rec, soff + (uint32_t)((kMetaWords + tile_words(KB)) * 4), l16, l8);
  }
};

__device__ __forceinline__ void st_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__device__ __forceinline__ half2_t as_half2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ uint32_t as_u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }
// Product of two fp16 pairs as packed fp16 pairs (hi, lo) with hi + lo == a * b to ~21 bits: hi is the product
// rounded to fp16 (one packed multiply), lo the residual of the exact product against that same register (one
// packed fused multiply-add; the residual of an fp16 product is itself an fp16 number unless it falls below
// 2^-24, where it is off by at most 2^-25 absolute).
__device__ __forceinline__ void mul_split(half2_t a, half2_t b, uint32_t& hi, uint32_t& lo) {
  const half2_t h = a * b;
  const half2_t l = __builtin_elementwise_fma(a, b, -h);
  hi = as_u32(h);
  lo = as_u32(l);
}
// fp32 pair -> packed fp16 pairs (hi, lo) with hi + lo == x to ~22 bits.
// The hi parts come from the truncating packed conversion, an intrinsic of its own: written as a plain
// cast, the multiply that produced x may get fused into one of the two uses of the hi part only, and the
// stored hi part and the one the lo part refers to then differ by a double rounding.
__device__ __forceinline__ void split_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  const half2_t hv = __builtin_bit_cast(half2_t, __builtin_amdgcn_cvt_pkrtz(x0, x1));
  const half_t l0 = (half_t)(x0 - (float)hv[0]), l1 = (half_t)(x1 - (float)hv[1]);
  const half2_t lv = {l0, l1};
  hi = __builtin_bit_cast(uint32_t, hv);
  lo = __builtin_bit_cast(uint32_t, lv);
}
__device__ __forceinline__ half_t split_part(float x, bool lo_part) {
  const half2_t hv = __builtin_bit_cast(half2_t, __builtin_amdgcn_cvt_pkrtz(x, 0.0f));
  const half_t hi = hv[0];
  const half_t lo = (half_t)(x - (float)hi);
  return lo_part ? lo : hi;
}
__device__ __forceinline__ float lo_half(uint32_t v) { return (float)__builtin_bit_cast(half_t, (uint16_t)(v & 0xffffu)); }
__device__ __forceinline__ float hi_half(uint32_t v) { return (float)__builtin_bit_cast(half_t, (uint16_t)(v >> 16)); }

// Wave-private LDS exchange area. Operand rows exist for the 2*G used MFMA columns only (row 2h holds the hi
// parts of head h, row 2h+1 its lo parts: neighbours, so that one two-address LDS write stores both); the lanes
// of unused columns all read an extra zero row.
// Row pitches (272 B, 80 B) put the rows read by one 16-byte operand load into distinct banks.
template <int G> struct __attribute__((aligned(16))) WaveLds {
  static constexpr int kRows = 2 * G;                 // index of the zero row (present when columns are unused)
  static constexpr int kZeroRow = kRows < 16 ? 1 : 0;
  uint16_t bk[kRows + kZeroRow][kD + 8];   // scale-folded query [row][channel]
  // zero-points of the tile: the Key ones [channel] while the Key side is worked on, then the Value ones
  // [channel block][token] (the same 256 bytes: the Key side is done with them before the Value ones are written)
  union { uint16_t zk[kD]; uint16_t zv[4][kTile]; };
  // scores of the tile [row][token] (rows as in bk). Pitch 144 B: the rows are written 16 bytes per lane by
  // the 16 columns at once, and with a pitch of 128 B all rows would start in the same banks (measured: the two
  // stores of a tile took as long as all its other LDS traffic together)
  float s[2 * G][kTile + 4];
  // scale-folded softmax numerators [channel block][row][token]; the four blocks, written together 4 bytes per
  // lane, start 64 bytes apart modulo the 256 bytes of one pass over the banks
  struct BvBlock { uint16_t r[kRows + kZeroRow][kTile + 8]; uint16_t pad[((kRows + kZeroRow) * (kTile + 8) * 2 % 256 == 64) ? 0 : (64 + 256 - (kRows + kZeroRow) * (kTile + 8) * 2 % 256) % 256 / 2]; };
  BvBlock bv[4];
  uint16_t pq[kRows + kZeroRow][kTile + 8];   // softmax numerators as two fp16 terms [row][token] (rows as in bk)
};

template <int G> struct MergeLds {        // per-wave reference maximum and sum of numerators of every head
  float m[waves_for(G)][G];
  float l[waves_for(G)][G];
};

template <int KB, int VB, int G>
__global__ __launch_bounds__(waves_for(G) * kWave) void decode_attn_kernel(AttnArgs a) {
  constexpr int kWaves = waves_for(G);
  constexpr int kThreads = kWaves * kWave;
  // per wave: the exchange area of the packed tiles; before that, the staging area in which a window tile's
  // Value rows (token-major in memory) are turned into matrix-core operands (8 consecutive tokens per lane)
  constexpr int kTPitch = kD + 8;   // fp16 elements per staged row (272 B: 16-byte aligned rows)
  // and, once the wave has worked through its tiles, its result (a wave's memory is its own: a wave that is
  // done never waits for the others)
  union WaveArea { WaveLds<G> x; uint16_t t[kTile][kTPitch]; float o[G][kD + 16]; };   // result rows 64 bytes apart modulo a pass over the banks
  __shared__ WaveArea s_wave[kWaves];
  __shared__ MergeLds<G> R;
  __shared__ int s_next;   // next unclaimed packed tile of this workgroup
  __shared__ int s_done;   // waves that have delivered their result

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // said to be uniform: what depends on it alone lives in scalar registers
  const int col = lane & 15, kq = lane >> 4;         // MFMA column / row index, k-quarter
  const int h = col & 7;
  const bool lo_part = col >= 8;
  const bool col_valid = h < G;
  const int sp = blockIdx.x, u = blockIdx.y;
  // Query groups of more than 8 heads run as blocks of 8 heads in workgroups of their own (grid z): the blocks of
  // a unit read the same records and window rows at about the same time, so a tile comes from HBM once and from
  // the caches after that. uo numbers the (unit, head block) pairs: rows uo*8 .. uo*8+7 of q and out.
  const int uo = u * (int)gridDim.z + (int)blockIdx.z;
  WaveLds<G>& L = s_wave[wave].x;
  uint16_t (&T)[kTile][kTPitch] = s_wave[wave].t;
  const int row = col_valid ? 2 * h + (lo_part ? 1 : 0) : WaveLds<G>::kRows;   // operand row of this lane's column

  // Work items of this split: window tiles first, then packed tiles. Split sp takes items_q items, the first
  // items_r splits one more (quotient and remainder come from the host: the start of a launch is latency-bound
  // and integer division takes hundreds of instructions here).
  const int n_wt = a.W_cap >> 5;
  const int item_begin = sp * a.items_q + (sp < a.items_r ? sp : a.items_r);
  const int item_end = item_begin + a.items_q + (sp < a.items_r ? 1 : 0);
  const int win_begin = item_begin < n_wt ? item_begin : n_wt;
  const int win_end = item_end < n_wt ? item_end : n_wt;
  const int p_begin = (item_begin > n_wt ? item_begin : n_wt) - n_wt;
  const int p_end = (item_end > n_wt ? item_end : n_wt) - n_wt;

  // ---- the query and the wave's first window tile are requested before anything else is done.
  // Packed tiles are claimed from a workgroup counter; the first claims are static (wave order).
  const uint16_t* qbase = a.q + (size_t)uo * (G * kD);   // heads of unit u = (b, j) are rows (b*Hkv + j)*G .. +G-1 of q and out
  half8_t qB[4];       // plain q as B operand: hi columns hold head h, everything else zero
  uint32_t qraw[G];    // q of channels (2*lane, 2*lane+1) of every head
  {
    const half8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      half8_t v = zero8;
      if (col_valid && !lo_part) v = *reinterpret_cast<const half8_t*>(qbase + (size_t)h * kD + 32 * ks + 8 * kq);
      qB[ks] = v;
    }
#pragma unroll
    for (int hh = 0; hh < G; hh++) qraw[hh] = reinterpret_cast<const uint32_t*>(qbase + (size_t)hh * kD)[lane];
  }

  // Fused append: the newest token of the unit is not in the window arrays yet. The wave that takes the window
  // tile of its ring slot reads that one row from k_new / v_new instead of the ring, treats it like any other
  // row of the tile (the host counts it in n_w) and stores it into the ring for the steps to come.
  const int new_tile = a.new_slot >= 0 ? (a.new_slot >> 5) : -1;
  const int new_tau = a.new_slot & 31;

  constexpr uint32_t kRecBytes = (uint32_t)(record_words(KB, VB) * 4);
  const rsrc_t up = make_rsrc(reinterpret_cast<const char*>(a.packed) + (size_t)u * a.tiles_cap * kRecBytes, (uint32_t)a.tiles_cap * kRecBytes);
  const int n_win = win_end - win_begin;
  const int n_early = n_win < kWaves ? kWaves - n_win : 0;      // waves n_win .. kWaves-1 start on packed tiles
  const bool has_packed = p_end > p_begin;
  const bool early = has_packed && wave >= n_win;
  Stage<KB, VB> st[kDepth];
  int it[kDepth];

  // window tile wi of the ring: the Key rows as MFMA A operands (rows = tokens), the Value rows as loaded:
  // 16-byte piece lane + 64*j of the tile's 8 KiB, i.e. token 4*j + kq, channels 8*col .. 8*col+7
  struct WinTile { half8_t Ak[2][4]; u32x4_t Vr[8]; };
  auto win_first = [&](int wi) { const int r = wi * kTile - a.w0; return r < 0 ? r + a.W_cap : r; };   // ring rank of the tile's first slot
  auto win_load = [&](int wi, WinTile& w) {
    const int slot0 = wi * kTile;
    const uint16_t* kw = a.k_win + ((size_t)u * a.W_cap + slot0) * kD;
    const uint16_t* kn = a.k_new + (size_t)u * kD;
    const bool has_new = wi == new_tile;      // wave-uniform
#pragma unroll
    for (int m = 0; m < 2; m++) {
      const int tau = 8 * (col >> 2) + 4 * m + (col & 3);   // row `col` of M-tile m
      // a slot past the live tokens is not read: its lanes take the tile's first row instead (live, and already on its
      // way: a cache hit), whose products the softmax mask discards; no byte of a dead slot reaches the arithmetic
      const int tau_r = win_first(wi) + tau < a.n_w ? tau : 0;
      const uint16_t* rowp = (has_new && tau == new_tau) ? kn : kw + (size_t)tau_r * kD;
#pragma unroll
      for (int ks = 0; ks < 4; ks++) w.Ak[m][ks] = *reinterpret_cast<const half8_t*>(rowp + 32 * ks + 8 * kq);
    }
  };
  // The Value rows are requested only when the Key rows have been consumed: fewer registers in flight (no
  // spills in any variant) and a smaller first burst, so that the first packed tiles arrive earlier
  // (measured 0.3-0.4 us per launch against requesting both at the start).
  auto win_load_v = [&](int wi, WinTile& w) {
    const uint16_t* vw = a.v_win + ((size_t)u * a.W_cap + wi * kTile) * kD;
    const uint16_t* vn = a.v_new + (size_t)u * kD;
    const bool has_new = wi == new_tile;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const int tv = win_first(wi) + 4 * j + kq < a.n_w ? 4 * j + kq : 0;      // dead slots: the first row again (weight zero)
      const uint16_t* rowp = (has_new && 4 * j + kq == new_tau) ? vn : vw + (size_t)tv * kD;
      w.Vr[j] = *reinterpret_cast<const u32x4_t*>(rowp + 8 * col);
    }
  };
  // the append itself: the lanes that hold pieces of the new row store them into its ring slot
  auto store_new_k = [&](int wi, const WinTile& w) {
    if (wi != new_tile) return;
    uint16_t* dst = a.k_win_w + ((size_t)u * a.W_cap + a.new_slot) * kD;
#pragma unroll
    for (int m = 0; m < 2; m++) {
      const int tau = 8 * (col >> 2) + 4 * m + (col & 3);
      if (tau == new_tau) {
#pragma unroll
        for (int ks = 0; ks < 4; ks++) *reinterpret_cast<half8_t*>(dst + 32 * ks + 8 * kq) = w.Ak[m][ks];
      }
    }
  };
  auto store_new_v = [&](int wi, const WinTile& w) {
    if (wi != new_tile) return;
    uint16_t* dst = a.v_win_w + ((size_t)u * a.W_cap + a.new_slot) * kD;
#pragma unroll
    for (int j = 0; j < 8; j++)
      if (4 * j + kq == new_tau) *reinterpret_cast<u32x4_t*>(dst + 8 * col) = w.Vr[j];
  };
  WinTile wt;
  int wi = win_begin + wave;
  // tiles wholly outside the n_w valid tokens are skipped (w0 and tiles are 32-aligned)
  while (wi < win_end && win_first(wi) >= a.n_w) wi += kWaves;
  if (wi < win_end) win_load(wi, wt);

  if (tid == 0) { s_next = p_begin + kDepth * n_early; s_done = 0; }
  // The only workgroup barrier before the results are merged: the counters are set. It must not wait for the
  // loads just requested (a full __syncthreads would): LDS serves a wave's operations in order, so waiting for
  // the wave's LDS operations before the barrier is all that the two counter writes need.
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");   // no memory access of the code below moves above the barrier

  // q of the lane's two channels, prescaled so that code products of all four channel blocks come out in the
  // same unit: the field of block ks sits at bit field_pos(ks), the query is scaled by 2^(field_pos(0) - field_pos(ks))
  // (exact in fp16 for |q| >= 2^-8; smaller values lose bits far below anything the scores resolve)
  constexpr int kPos0 = field_pos<KB>(0);
  half2_t qh[G];
  {
    const half_t pre = (half_t)__builtin_ldexpf(1.0f, kPos0 - field_pos<KB>(lane >> 4));
#pragma unroll
    for (int hh = 0; hh < G; hh++) qh[hh] = as_half2(qraw[hh]) * half2_t{pre, pre};
  }

  const half8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  const half8_t ones8 = {1, 1, 1, 1, 1, 1, 1, 1};
  const float c_code = a.scale_log2 * __builtin_ldexpf(1.0f, 24 - kPos0);   // code products carry 2^(field_pos(0) - 24)
  const float c_plain = a.scale_log2;

  float4_t acc[8];
  float4_t accZ = {0, 0, 0, 0};
#pragma unroll
  for (int m = 0; m < 8; m++) acc[m] = float4_t{0, 0, 0, 0};
  float mref = -INFINITY;

  // online softmax of the lane's 8 tokens (8*kq + e of the tile, column col). The score of token e is
  // s[e]*c + z (log2 domain) summed over the hi and lo columns; z is zero in lo columns. Raises the
  // reference if needed (rescaling the accumulators) and returns the numerators 2^(score - reference).
  // raises the per-column reference to cover mx (log2-domain upper estimate of the tile's scores,
  // identical in all lanes of a column pair) and rescales the accumulators accordingly
  auto raise_reference = [&](float mx) {
    if (__any(mx > mref + kRefCap)) {
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = mx > mref + kRefCap ? mx + kRefMargin : mref;
      const float f = (mnew == mref) ? 1.0f : fast_exp2(mref - mnew);
      mref = mnew;
      accZ *= f;
#pragma unroll
      for (int m = 0; m < 8; m++) acc[m] *= f;
    }
  };
  auto max8 = [](const float (&s)[8]) {
    float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
    mx = fmaxf(fmaxf(mx, s[3]), s[4]);
    mx = fmaxf(fmaxf(mx, s[5]), s[6]);
    return fmaxf(mx, s[7]);
  };

  // claiming a tile: the counter update is issued early (lane 0) and its result taken after the tile in
  // between has been worked on, so that the LDS round trip is not waited for
  auto grab_issue = [&]() -> int {
    int t = 0;
    if (lane == 0) t = __hip_atomic_fetch_add(&s_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return t;
  };
  auto grab_take = [](int t) -> int { return __builtin_amdgcn_readfirstlane(t); };
  auto grab = [&]() -> int { return grab_take(grab_issue()); };

  // ---- fp16 window tiles (few): taken round-robin by the waves before the packed stream.
  // A wave that started on packed tiles has no window tile; the nesting keeps its tile registers
  // out of the live ranges in here.
  if (!early) {
  while (wi < win_end) {
    const int first = win_first(wi);
    const half8_t (&Ak)[2][4] = wt.Ak;
    float4_t S[2] = {float4_t{0, 0, 0, 0}, float4_t{0, 0, 0, 0}};
#pragma unroll
    for (int m = 0; m < 2; m++)
#pragma unroll
      for (int ks = 0; ks < 4; ks++) S[m] = mfma16(Ak[m][ks], qB[ks], S[m]);
    store_new_k(wi, wt);
    win_load_v(wi, wt);
    // Value rows into the staging area as loaded (their registers are free again before the softmax). Rows
    // 16..31 swap neighbouring 32-byte blocks, so that the lanes of different kq read from different banks.
#pragma unroll
    for (int j = 0; j < 8; j++) *reinterpret_cast<u32x4_t*>(&T[4 * j + kq][8 * (col ^ (j >= 4 ? 2 : 0))]) = wt.Vr[j];
    store_new_v(wi, wt);
    float x[8], p[8];
#pragma unroll
    for (int m = 0; m < 2; m++)
#pragma unroll
      for (int r = 0; r < 4; r++) x[4 * m + r] = (first + 8 * kq + 4 * m + r) < a.n_w ? S[m][r] : -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; e++) x[e] = x[e] + ror8(x[e]);   // hi column + lo column (lo is zero here)
    raise_reference(max8(x) * c_plain);
#pragma unroll
    for (int e = 0; e < 8; e++) p[e] = fast_exp2(x[e] * c_plain - mref);
    half8_t PB;
#pragma unroll
    for (int e = 0; e < 8; e++) PB[e] = split_part(col_valid ? p[e] : 0.0f, lo_part);
    accZ = mfma16(col >= 4 ? ones8 : zero8, PB, accZ);   // rows 4..15 accumulate the sum of numerators
    // Value rows back from the staging area, channel by channel
    wave_lds_fence();
#pragma unroll
    for (int m = 0; m < 8; m++) {
      half8_t Avm;
#pragma unroll
      for (int e = 0; e < 8; e++) Avm[e] = __builtin_bit_cast(half_t, T[8 * kq + e][16 * (m ^ (kq >> 1)) + col]);
      float4_t t = mfma16(Avm, PB, float4_t{0, 0, 0, 0});
      if constexpr (VB == 3) {   // the final 7/3 step factor of channels 10 / 21 applies to codes only
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int dd = 16 * (m & 1) + 4 * kq + r;
          if (dd == 10 || dd == 21) t[r] *= (3.0f / 7.0f);
        }
      }
      acc[m] += t * __builtin_ldexpf(1.0f, field_pos<VB>(m & 3) - 24);
    }
    wave_lds_fence();   // the staging area is free again
    wi += kWaves;
    while (wi < win_end && win_first(wi) >= a.n_w) wi += kWaves;
    if (wi < win_end) win_load(wi, wt);
  }
  if (has_packed) {   // claim the first packed tiles now
#pragma unroll
    for (int s = 0; s < kDepth; s++) {
      it[s] = grab();
      st[s].load(up, it[s] < p_end ? it[s] : p_end - 1, lane);
    }
  }
  }
  // The waves without a window tile take their first packed tiles by wave order (the counter starts behind
  // them). They request them only here, not at the kernel's start: tile registers that stay live across the
  // window code above push the kernel over its register budget, and the spill that follows waits for every
  // outstanding load; requested here they cost nothing measurable (the start of a launch is bound by the
  // request rate of the window and query loads anyway).
  // Past the end a wave re-reads the last tile (cache hit) and skips its work: the load stream and the
  // loop body stay uniform, which keeps the outstanding-load accounting exact.
  if (early) {
#pragma unroll
    for (int s = 0; s < kDepth; s++) {
      it[s] = p_begin + s * n_early + (wave - n_win);
      st[s].load(up, it[s] < p_end ? it[s] : p_end - 1, lane);
    }
  }

  // zero the wave's exchange area (it shared its memory with the staging area): the rows of unused
  // operand columns stay zero from here on
  {
    u32x4_t* z = reinterpret_cast<u32x4_t*>(&L);
    for (int i = lane; i < (int)(sizeof(WaveLds<G>) / 16); i += kWave) z[i] = u32x4_t{0, 0, 0, 0};
  }
  wave_lds_fence();

  // ---- small query groups (G <= 2): the matrix core's columns are nearly empty, so the per-tile extras
  // (Key zero-point term, Value zero-point term, sum of numerators) are cheaper on the vector unit:
  // a packed dot product plus a wave reduction, and per-lane running sums reduced once at the end.
  constexpr bool kSmall = G <= 2;
  float lwin = 0.0f;            // window tiles' sum of numerators of the lane's column (hi + lo)
  float lacc[G], zacc[G];       // running sum of numerators / of numerator * Value minimum over the lane's tokens
  float mref_u[G];              // reference of head hh, the same value in every lane
  if constexpr (kSmall) {
    lwin = __shfl(accZ[0], 16 + col);
    lwin += ror8(lwin);
#pragma unroll
    for (int hh = 0; hh < G; hh++) {
      lacc[hh] = 0.0f; zacc[hh] = 0.0f;
      mref_u[hh] = uniform_lane(mref, hh);
    }
  }
  const float inv_c_code = 1.0f / c_code;

  auto process_small = [&](const Stage<KB, VB>& st) {
    // -- Key side. Lane owns channels 2*lane, 2*lane+1: scale-folded query to LDS, zero-point term by dot product
    float zt[G];
    {
      const half2_t s2 = as_half2(st.meta[0]);
      const uint32_t kz_pair = st.meta[1];   // a copy: a bit cast applied to the vector element itself reads element 0
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        uint32_t hi, lo;
        mul_split(qh[hh], s2, hi, lo);
        reinterpret_cast<uint32_t*>(&L.bk[2 * hh][0])[lane] = hi;
        reinterpret_cast<uint32_t*>(&L.bk[2 * hh + 1][0])[lane] = lo;
        const float zp = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, qraw[hh]), __builtin_bit_cast(half2_t, kz_pair), 0.0f, false);
        zt[hh] = wave_sum(zp) * c_plain;
      }
    }
    wave_lds_fence();
    {
      const Codes<KB> kc(st.kc);
      half8_t Bk[4];
#pragma unroll
      for (int ks = 0; ks < 4; ks++) Bk[ks] = *reinterpret_cast<const half8_t*>(&L.bk[row][32 * ks + 8 * kq]);
      float4_t S[2] = {float4_t{0, 0, 0, 0}, float4_t{0, 0, 0, 0}};
#pragma unroll
      for (int m = 0; m < 2; m++)
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
          S[m] = mfma16(kc.lo(ks + 4 * m), Bk[ks], S[m]);
        }
      if constexpr (KB == 3) {   // tokens 10 and 21 of the group step by s*7/3
        if (kq == 1) S[0][2] *= (7.0f / 3.0f);
        if (kq == 2) S[1][1] *= (7.0f / 3.0f);
      }
      if (col_valid) {
        *reinterpret_cast<float4_t*>(&L.s[row][8 * kq]) = S[0];
        *reinterpret_cast<float4_t*>(&L.s[row][8 * kq + 4]) = S[1];
      }
    }
    wave_lds_fence();
    // -- Value side. Lane (tp, g) owns tokens (2*tp, 2*tp+1) of channel block g.
    {
      const int tp = lane & 15, g = lane >> 4;
      const float s0 = lo_half(st.meta[2]), s1 = hi_half(st.meta[2]);
      const float z0 = lo_half(st.meta[3]), z1 = hi_half(st.meta[3]);
      float sum0[G], sum1[G];
      bool over = false;
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        const float2_t sh = *reinterpret_cast<const float2_t*>(&L.s[2 * hh][2 * tp]);
        const float2_t sl = *reinterpret_cast<const float2_t*>(&L.s[2 * hh + 1][2 * tp]);
        sum0[hh] = sh[0] + sl[0];
        sum1[hh] = sh[1] + sl[1];
        // score = sum * c_code + zt; it exceeds what the reference allows iff sum > (reference + cap - zt) / c_code
        over |= fmaxf(sum0[hh], sum1[hh]) > (mref_u[hh] + kRefCap - zt[hh]) * inv_c_code;
      }
      if (__any(over)) {   // rare: raise the reference of the heads that need it and rescale what was accumulated
#pragma unroll
        for (int hh = 0; hh < G; hh++) {
          const float mx = wave_max(fmaxf(sum0[hh], sum1[hh])) * c_code + zt[hh];
          if (mx > mref_u[hh] + kRefCap) {          // wave-uniform
            const float mnew = mx + kRefMargin;
            const float f = fast_exp2(mref_u[hh] - mnew);      // 0 for the first tile (reference -inf)
            mref_u[hh] = mnew;
            lacc[hh] *= f; zacc[hh] *= f;
            if (h == hh) {                // the lanes of this head's columns
              mref = mnew;
              lwin *= f;
#pragma unroll
              for (int m = 0; m < 8; m++) acc[m] *= f;
            }
          }
        }
      }
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        const float off = zt[hh] - mref_u[hh];
        const float p0 = fast_exp2(sum0[hh] * c_code + off);
        const float p1 = fast_exp2(sum1[hh] * c_code + off);
        lacc[hh] += p0 + p1;
        zacc[hh] += p0 * z0 + p1 * z1;
        uint32_t hi, lo;
        split_pair(p0 * s0, p1 * s1, hi, lo);
        reinterpret_cast<uint32_t*>(&L.bv[g].r[2 * hh][0])[tp] = hi;
        reinterpret_cast<uint32_t*>(&L.bv[g].r[2 * hh + 1][0])[tp] = lo;
      }
    }
    wave_lds_fence();
    {
      const Codes<VB> vc(st.vc);
      half8_t Bv[4];
#pragma unroll
      for (int g = 0; g < 4; g++) Bv[g] = *reinterpret_cast<const half8_t*>(&L.bv[g].r[row][8 * kq]);
#pragma unroll
      for (int m = 0; m < 8; m++) {
        acc[m] = mfma16(vc.lo(m), Bv[m >> 1], acc[m]);
      }
    }
    wave_lds_fence();   // the next tile's operand writes come after these reads
  };

  auto process_large = [&](const Stage<KB, VB>& st) {
    // -- Key side. Cooperative operand preparation: lane owns channels 2*lane, 2*lane+1.
    {
      const half2_t s2 = as_half2(st.meta[0]);
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        uint32_t hi, lo;
        mul_split(qh[hh], s2, hi, lo);
        reinterpret_cast<uint32_t*>(&L.bk[2 * hh][0])[lane] = hi;
        reinterpret_cast<uint32_t*>(&L.bk[2 * hh + 1][0])[lane] = lo;
      }
      reinterpret_cast<uint32_t*>(&L.zk[0])[lane] = st.meta[1];
    }
    wave_lds_fence();
    float x[8], zt;
    {
      const Codes<KB> kc(st.kc);
      half8_t Bk[4];
      float4_t Sz = {0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        Bk[ks] = *reinterpret_cast<const half8_t*>(&L.bk[row][32 * ks + 8 * kq]);
        const half8_t z8 = *reinterpret_cast<const half8_t*>(&L.zk[32 * ks + 8 * kq]);
        Sz = mfma16(z8, qB[ks], Sz);     // every A row is the zero-point vector
      }
      float4_t S[2] = {float4_t{0, 0, 0, 0}, float4_t{0, 0, 0, 0}};
#pragma unroll
      for (int m = 0; m < 2; m++)
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
          S[m] = mfma16(kc.lo(ks + 4 * m), Bk[ks], S[m]);
        }
      if constexpr (KB == 3) {   // tokens 10 and 21 of the group step by s*7/3
        if (kq == 1) S[0][2] *= (7.0f / 3.0f);
        if (kq == 2) S[1][1] *= (7.0f / 3.0f);
      }
      zt = Sz[0] * c_plain;          // zero in lo columns (their plain-query operand is zero)
#pragma unroll
      for (int m = 0; m < 2; m++)
#pragma unroll
        for (int r = 0; r < 4; r++) x[4 * m + r] = S[m][r];
    }
    // Reference maximum from the hi column (the lo column changes a score by < 2^-10 of its size, which a
    // reference does not need); lo lanes take their partner's value so that a column pair stays in step.
    float mx = max8(x) * c_code + zt;
    const float mx_partner = ror8(mx);        // cross-lane read outside any divergent branch: all lanes must take part
    mx = lo_part ? mx_partner : mx;
    raise_reference(mx);
    // log2-domain scores against the reference; the zero-point term and the reference enter through the hi column
    const float off_col = lo_part ? 0.0f : zt - mref;
#pragma unroll
    for (int e = 0; e < 8; e++) x[e] = x[e] * c_code + off_col;

    // -- Value side. Scores to LDS; lane (tp, g) then owns tokens (2*tp, 2*tp+1) of channel block g.
    if (col_valid) {
      *reinterpret_cast<float4_t*>(&L.s[row][8 * kq]) = float4_t{x[0], x[1], x[2], x[3]};
      *reinterpret_cast<float4_t*>(&L.s[row][8 * kq + 4]) = float4_t{x[4], x[5], x[6], x[7]};
    }
    wave_lds_fence();
    // The four lane groups g would all compute the same numerators; instead group g finishes those of the
    // heads 4k + g only and hands them to the others through LDS as two fp16 terms (the rounded value and what
    // the rounding left over: together ~22 bits, the same pair enters the Value sums, the zero-point sums and
    // the denominator).
    {
      const int tp = lane & 15, g = lane >> 4;
      // (all reads of a step are issued before its first write: the compiler does not move LDS reads across LDS
      // writes through pointers of the same type, and one read at a time costs an LDS round trip each)
      constexpr int kShare = G / 4 > 0 ? G / 4 : 1;   // (the function is only used with groups of 4 or 8 heads)
      float2_t sh[kShare], sl[kShare];
#pragma unroll
      for (int k = 0; k < G / 4; k++) {
        const int hh = 4 * k + g;                                  // differs between the lane groups
        sh[k] = *reinterpret_cast<const float2_t*>(&L.s[2 * hh][2 * tp]);
        sl[k] = *reinterpret_cast<const float2_t*>(&L.s[2 * hh + 1][2 * tp]);
      }
#pragma unroll
      for (int k = 0; k < G / 4; k++) {
        const int hh = 4 * k + g;
        // leading terms rounded to nearest: they are multiplied on their own below, and a truncated leading term
        // whose remainder's product falls below the fp16 range would bias the sums (plain casts are safe here:
        // the values come out of the exponential instruction, nothing can be fused into the conversions)
        const float p0 = fast_exp2(sh[k][0] + sl[k][0]), p1 = fast_exp2(sh[k][1] + sl[k][1]);
        const half2_t hv = {(half_t)p0, (half_t)p1};
        const half2_t lv = {(half_t)(p0 - (float)hv[0]), (half_t)(p1 - (float)hv[1])};
        reinterpret_cast<uint32_t*>(&L.pq[2 * hh][0])[tp] = as_u32(hv);
        reinterpret_cast<uint32_t*>(&L.pq[2 * hh + 1][0])[tp] = as_u32(lv);
      }
      reinterpret_cast<uint32_t*>(&L.zv[0][0])[lane] = st.meta[3];
    }
    wave_lds_fence();
    {
      const int tp = lane & 15, g = lane >> 4;
      const half2_t s2 = as_half2(st.meta[2]);
      uint32_t pw[G], dw[G];
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        pw[hh] = reinterpret_cast<const uint32_t*>(&L.pq[2 * hh][0])[tp];
        dw[hh] = reinterpret_cast<const uint32_t*>(&L.pq[2 * hh + 1][0])[tp];
      }
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        const half2_t p2 = as_half2(pw[hh]), d2 = as_half2(dw[hh]);
        // (p2 + d2) * s2: exact product of the leading term in two parts, the small term's product folded into the second
        const half2_t hv = p2 * s2;
        const half2_t lv = __builtin_elementwise_fma(d2, s2, __builtin_elementwise_fma(p2, s2, -hv));
        reinterpret_cast<uint32_t*>(&L.bv[g].r[2 * hh][0])[tp] = as_u32(hv);
        reinterpret_cast<uint32_t*>(&L.bv[g].r[2 * hh + 1][0])[tp] = as_u32(lv);
      }
    }
    wave_lds_fence();
    {
      const Codes<VB> vc(st.vc);
      half8_t Bv[4];
#pragma unroll
      for (int g = 0; g < 4; g++) Bv[g] = *reinterpret_cast<const half8_t*>(&L.bv[g].r[row][8 * kq]);
      // plain numerators: the column's own row (unused columns: the zero row)
      const half8_t PB = *reinterpret_cast<const half8_t*>(&L.pq[row][8 * kq]);
      // zero-point term: A rows 0..3 carry the zero-points of channel blocks 0..3, rows 4..15 are ones
      // and accumulate the sum of the numerators
      half8_t z8 = ones8;
      if (col < 4) z8 = *reinterpret_cast<const half8_t*>(&L.zv[col][8 * kq]);
      accZ = mfma16(z8, PB, accZ);
#pragma unroll
      for (int m = 0; m < 8; m++) {
        acc[m] = mfma16(vc.lo(m), Bv[m >> 1], acc[m]);
      }
    }
    wave_lds_fence();   // the next tile's operand writes come after these reads
  };
  auto process = [&](const Stage<KB, VB>& st) {
    if constexpr (kSmall) process_small(st); else process_large(st);
  };

  if (has_packed) {
    while (it[0] < p_end) {      // a wave's items increase: it[0] is the oldest one in flight
#pragma unroll
      for (int s = 0; s < kDepth; s++) {
        const int ticket = grab_issue();
        if (it[s] < p_end) process(st[s]);   // past the end: skip the work, keep the load stream
        const int nxt = grab_take(ticket);
        it[s] = nxt;
        st[s].load(up, nxt < p_end ? nxt : p_end - 1, lane);
      }
    }
  }

  // ---- per-wave result (into the wave's own area, whose exchange contents are no longer needed): undo the
  // field scaling, add hi and lo columns, add the zero-point term.
  // accZ: lanes with kq == 0 hold the zero-point sums of channel blocks 0..3, lanes with kq >= 1 the
  // sum of numerators (any register).
  float zsum[4];
  float lsum;
  if constexpr (kSmall) {
    // running sums: the lanes of row 0 cover all tokens once (numerators), the lanes of row g hold the
    // zero-point sums of channel block g; hi lanes take the whole term, lo lanes nothing
    lsum = lwin;
#pragma unroll
    for (int g = 0; g < 4; g++) zsum[g] = 0.0f;
#pragma unroll
    for (int hh = 0; hh < G; hh++) {
      const float lr = row_sum(lacc[hh]), zr = row_sum(zacc[hh]);
      const bool mine = col == hh;
      const float lt = uniform_lane(lr, 0);   // cross-lane reads stay outside divergent code: the source lane must be active
      lsum += mine ? lt : 0.0f;
#pragma unroll
      for (int g = 0; g < 4; g++) { const float t = uniform_lane(zr, 16 * g); zsum[g] = mine ? t : zsum[g]; }
    }
  } else {
#pragma unroll
    for (int g = 0; g < 4; g++) zsum[g] = __shfl(accZ[g], col);
    lsum = __shfl(accZ[0], 16 + col);
    lsum += ror8(lsum);
  }
#pragma unroll
  for (int m = 0; m < 8; m++) {
    const float sc = __builtin_ldexpf(1.0f, 24 - field_pos<VB>(m & 3));
    float4_t o4;
#pragma unroll
    for (int r = 0; r < 4; r++) {
      float v = acc[m][r] * sc;
      if (VB == 3) {   // channels 10 and 21 of each block of 32 step by s*7/3
        const int dd = 16 * (m & 1) + 4 * kq + r;
        if (dd == 10 || dd == 21) v *= (7.0f / 3.0f);
      }
      v += zsum[m >> 1];
      o4[r] = v + ror8(v);
    }
    if (col < G) *reinterpret_cast<float4_t*>(&s_wave[wave].o[col][16 * m + 4 * kq]) = o4;   // channels 16m + 4kq .. +3
  }
  if (col < G && kq == 0) { R.m[wave][col] = mref; R.l[wave][col] = lsum; }

  // combines the per-wave results of output idx = head * 128 + channel
  auto combine = [&](int idx, float& M, float& Lsum, float& O) {
    const int hh = idx / kD, d = idx % kD;
    M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; w++) M = fmaxf(M, R.m[w][hh]);
    Lsum = 0.0f; O = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; w++) {
      const float mw = R.m[w][hh];
      const float f = (mw == -INFINITY) ? 0.0f : fast_exp2(mw - M);
      Lsum += R.l[w][hh] * f;
      O += s_wave[w].o[hh][d] * f;
    }
  };
  uint16_t* outp = a.out + (size_t)uo * (G * kD);

  if (a.n_parts == 1) {
    if constexpr (G <= 2) {
      // No barrier: a wave delivers its result and leaves; the last one to deliver combines them.
      // (LDS serves a wave's operations in order, so its results are in place before its count.)
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      int done = 0;
      if (lane == 0) done = __hip_atomic_fetch_add(&s_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      done = __builtin_amdgcn_readfirstlane(done);
      if (done != kWaves - 1) return;
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      // lane w < kWaves holds wave w's reference and sum; the weights 2^(m_w - M) are computed once per head
      // and handed out as scalars, then every lane adds up two channels over the waves
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        const bool has = lane < kWaves;
        const float mw = has ? R.m[has ? lane : 0][hh] : -INFINITY;
        const float lw = has ? R.l[has ? lane : 0][hh] : 0.0f;
        float o0[kWaves], o1[kWaves];         // requested first: their latency overlaps the weight computation
#pragma unroll
        for (int w = 0; w < kWaves; w++) { o0[w] = s_wave[w].o[hh][lane]; o1[w] = s_wave[w].o[hh][lane + kWave]; }
        const float M = uniform_lane(row_max(mw), 0);
        const float fw = (mw == -INFINITY) ? 0.0f : fast_exp2(mw - M);
        const float Lsum = uniform_lane(row_sum(lw * fw), 0);
        float O0 = 0.0f, O1 = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; w++) {
          const float f = uniform_lane(fw, w);
          O0 += o0[w] * f;
          O1 += o1[w] * f;
        }
        const float inv = 1.0f / Lsum;
        outp[hh * kD + lane] = __builtin_bit_cast(uint16_t, (half_t)(O0 * inv));
        outp[hh * kD + lane + kWave] = __builtin_bit_cast(uint16_t, (half_t)(O1 * inv));
      }
    } else {
      __syncthreads();
      for (int idx = tid; idx < G * kD; idx += kThreads) {
        float M, Lsum, O;
        combine(idx, M, Lsum, O);
        outp[idx] = __builtin_bit_cast(uint16_t, (half_t)(O / Lsum));
      }
    }
    return;
  }

  __syncthreads();
  for (int idx = tid; idx < G * kD; idx += kThreads) {
    float M, Lsum, O;
    combine(idx, M, Lsum, O);
    // agent-scope stores: written through to the level all XCDs share (no cache-wide flush needed)
    const int hh = idx / kD, d = idx % kD;
    float* pp = a.part + (((size_t)uo * a.n_parts + sp) * G + hh) * (kD + 2);
    if (d == 0) { st_agent(pp, M); st_agent(pp + 1, Lsum); }
    st_agent(pp + 2 + d, O);
  }

  // ---- split merge: the last workgroup of the unit to arrive combines all partials (n_parts of them: one per
  // split, and the one an earlier launch may have left for the tokens between a Key front and a Value front)
  // The partials were stored and are later loaded with agent scope, which the hardware keeps coherent
  // per access across the XCDs' L2s: waiting for the stores to complete is all the release needs.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's partial stores have completed ...
  __syncthreads();                                     // ... and so have those of all waves, before the arrival is counted
  if (tid == 0) {
    const uint32_t prev = __hip_atomic_fetch_add(&a.counters[uo], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_done = (prev == (uint32_t)a.n_splits - 1u);   // reused as the "last workgroup" flag
  }
  __syncthreads();
  if (!s_done) return;
  for (int idx = tid; idx < G * kD; idx += kThreads) {
    const int hh = __builtin_amdgcn_readfirstlane(idx / kD), d = idx % kD;   // a wave's 64 outputs share the head
    const float* base = a.part + ((size_t)uo * a.n_parts * G + hh) * (kD + 2);
    const size_t stride = (size_t)G * (kD + 2);
    // one pass, kMergeBatch partials per round trip: lane k requests reference and sum of the batch's k-th
    // partial, every lane its channel of each of them, all before the first use; the weights 2^(m_k - M) are
    // computed once per wave (lane k holds the k-th) and handed out as scalars
    float M = -INFINITY, Lsum = 0.0f, O = 0.0f;
    for (int s0 = 0; s0 < a.n_parts; s0 += kMergeBatch) {
      float mk = -INFINITY, lk = 0.0f;
      if (lane < kMergeBatch && s0 + lane < a.n_parts) {
        const float* pp = base + (size_t)(s0 + lane) * stride;
        mk = ld_agent(pp);
        lk = ld_agent(pp + 1);
      }
      float os[kMergeBatch];
#pragma unroll
      for (int k = 0; k < kMergeBatch; k++) {
        os[k] = 0.0f;
        if (s0 + k < a.n_parts) os[k] = ld_agent(base + (size_t)(s0 + k) * stride + 2 + d);   // wave-uniform test
      }
      // cross-lane reads stay outside divergent code
      const float mrow = row_max(mk);
      const float Mn = fmaxf(M, fmaxf(uniform_lane(mrow, 0), uniform_lane(mrow, 16)));
      const float fold = (M == -INFINITY) ? 0.0f : fast_exp2(M - Mn);
      const float fk = (mk == -INFINITY) ? 0.0f : fast_exp2(mk - Mn);
      const float lrow = row_sum(lk * fk);
      Lsum = Lsum * fold + (uniform_lane(lrow, 0) + uniform_lane(lrow, 16));
      O *= fold;
#pragma unroll
      for (int k = 0; k < kMergeBatch; k++) O += os[k] * uniform_lane(fk, k);
      M = Mn;
    }
    outp[idx] = __builtin_bit_cast(uint16_t, (half_t)(O / Lsum));
  }
  if (tid == 0) __hip_atomic_store(&a.counters[uo], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int KB, int VB>
hipError_t launch_g(const AttnArgs& a, int G, dim3 grid, hipStream_t s) {
  switch (G) {
    case 1: decode_attn_kernel<KB, VB, 1><<<grid, waves_for(1) * kWave, 0, s>>>(a); break;
    case 2: decode_attn_kernel<KB, VB, 2><<<grid, waves_for(2) * kWave, 0, s>>>(a); break;
    case 4: decode_attn_kernel<KB, VB, 4><<<grid, waves_for(4) * kWave, 0, s>>>(a); break;
    case 8: decode_attn_kernel<KB, VB, 8><<<grid, waves_for(8) * kWave, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_attn(const AttnArgs& a, int k_bits, int v_bits, int G, int units, hipStream_t s) {
  const int head_blocks = G > 8 ? G / 8 : 1;
  if (G > 8) G = 8;
  const dim3 grid(a.n_splits, units, head_blocks);
  switch (k_bits * 10 + v_bits) {
    case 11: return launch_g<1, 1>(a, G, grid, s);
    case 12: return launch_g<1, 2>(a, G, grid, s);
    case 13: return launch_g<1, 3>(a, G, grid, s);
    case 14: return launch_g<1, 4>(a, G, grid, s);
    case 21: return launch_g<2, 1>(a, G, grid, s);
    case 31: return launch_g<3, 1>(a, G, grid, s);
    case 41: return launch_g<4, 1>(a, G, grid, s);
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
