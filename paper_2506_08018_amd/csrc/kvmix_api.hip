// C-ABI entry points of libkvmix: host-side validation and launch plumbing only.
// Contract and layout: include/kvmix.h.
#include <atomic>
#include <cmath>
#include <mutex>
#include "kvmix_common.hpp"

using namespace kvmix;

namespace {

std::atomic<int> g_last_hip_error{0};

constexpr int kMaxDevices = 64;

// Compute units of the current device, asked once per device (0 when the query fails).
int num_cus() {
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return 0;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

int hip_fail(hipError_t e) {
  g_last_hip_error.store((int)e);
  return KVMIX_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape_cfg(const kvmix_shape* sh, const kvmix_layer_cfg* cfg) {
  if (!sh || !cfg) return KVMIX_ERR_NULL;
  if (sh->group != kTile) return KVMIX_ERR_BAD_GROUP;
  if (sh->D != kD || sh->B < 1 || sh->Hkv < 1 || sh->Hq < 1 || sh->Hq % sh->Hkv) return KVMIX_ERR_BAD_SHAPE;
  const int G = sh->Hq / sh->Hkv;
  if (G != 1 && G != 2 && G != 4 && (G % 8 != 0 || G > 512)) return KVMIX_ERR_BAD_SHAPE;
  if ((long long)sh->B * sh->Hkv > 65535) return KVMIX_ERR_BAD_SHAPE;
  const int kb = cfg->k_bits, vb = cfg->v_bits;
  if (kb == 16 || vb == 16) {
    if (kb != 16 || vb != 16) return KVMIX_ERR_BAD_BITS;
  } else if (kb < 1 || kb > 4 || vb < 1 || vb > 4) {
    return KVMIX_ERR_BAD_BITS;
  }
  if (cfg->window != -1 && (cfg->window < 0 || cfg->window % kTile)) return KVMIX_ERR_BAD_SHAPE;
  return KVMIX_OK;
}

// ring slot of token t (both windows)
int slot_of(const kvmix_layer_cache* c, long long t) {
  long long s = (c->w0 + t - c->n_q) % c->W_cap;
  return (int)(s < 0 ? s + c->W_cap : s);
}
// tokens that live in the ring: from the older of the two fronts to the newest
int ring_tokens(const kvmix_layer_cache* c) { return c->n_w + (c->v_lead < 0 ? -c->v_lead : 0); }

int check_cache(const kvmix_layer_cfg* cfg, const kvmix_layer_cache* c, bool need_packed) {
  if (!c) return KVMIX_ERR_NULL;
  if (c->T_cap < 0 || c->T_cap % kTile || c->W_cap < kTile || c->W_cap % kTile) return KVMIX_ERR_BAD_SHAPE;
  if (c->n_q < 0 || c->n_q % kTile || c->n_q > c->T_cap) return KVMIX_ERR_BAD_SHAPE;
  if (c->n_w < 0 || c->n_w > c->W_cap || c->w0 < 0 || c->w0 >= c->W_cap || c->w0 % kTile) return KVMIX_ERR_BAD_SHAPE;
  if (c->v_lead > c->n_w || (long long)c->n_q + c->v_lead < 0 || (long long)c->n_w - c->v_lead > c->W_cap || (long long)c->n_q + c->v_lead > c->T_cap)
    return KVMIX_ERR_BAD_SHAPE;
  if (c->v_lead != 0 && cfg->k_bits == 16) return KVMIX_ERR_BAD_BITS;
  if (!c->k_win || !c->v_win) return KVMIX_ERR_NULL;
  if (!aligned16(c->k_win) || !aligned16(c->v_win)) return KVMIX_ERR_ALIGN;
  if (cfg->k_bits == 16) return c->n_q == 0 ? KVMIX_OK : KVMIX_ERR_BAD_BITS;
  if (need_packed || c->n_q > 0) {
    if (!c->packed) return KVMIX_ERR_NULL;
    if (!aligned16(c->packed)) return KVMIX_ERR_ALIGN;
    // a unit's records are addressed with 32-bit byte offsets
    if ((long long)(c->T_cap / kTile) * record_words(cfg->k_bits, cfg->v_bits) * 4 > 0x7fffffffLL) return KVMIX_ERR_BAD_SHAPE;
  }
  return KVMIX_OK;
}

// (unit, block of at most 8 query heads) pairs: each is one workgroup per split
int out_units(const kvmix_shape* sh) {
  const int G = sh->Hq / sh->Hkv;
  return sh->B * sh->Hkv * (G > 8 ? G / 8 : 1);
}

int max_splits(const kvmix_shape* sh) {
  const int units = out_units(sh);
  int s = 512 / units;
  if (s < 8) s = 8;
  if (s > 64) s = 64;
  return s;
}

size_t counters_bytes(int units) { return (((size_t)units * 4 + 255) / 256) * 256; }

void fill_quant_dst(QuantArgs& a, const kvmix_layer_cache* c) {
  a.packed = c->packed;
  a.tiles_cap = c->T_cap / kTile;
}

}  // namespace

extern "C" {

int kvmix_version(void) { return 1; }

const char* kvmix_strerror(int status) {
  switch (status) {
    case KVMIX_OK: return "ok";
    case KVMIX_ERR_NULL: return "null pointer";
    case KVMIX_ERR_BAD_BITS: return "unsupported bit-width";
    case KVMIX_ERR_BAD_GROUP: return "unsupported group size";
    case KVMIX_ERR_BAD_SHAPE: return "unsupported shape or count";
    case KVMIX_ERR_ALIGN: return "misaligned pointer or stride";
    case KVMIX_ERR_WORKSPACE: return "workspace too small";
    case KVMIX_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

int kvmix_last_hip_error(void) { return g_last_hip_error.load(); }

int kvmix_cache_bytes(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, int T_cap, int W_cap,
                      size_t* packed_b, size_t* win_b) {
  const int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (T_cap < 0 || T_cap % kTile || W_cap < kTile || W_cap % kTile) return KVMIX_ERR_BAD_SHAPE;
  const size_t units = (size_t)sh->B * sh->Hkv, tiles = (size_t)T_cap / kTile;
  const bool packed = cfg->k_bits != 16;
  if (packed_b) *packed_b = packed ? units * tiles * record_words(cfg->k_bits, cfg->v_bits) * 4 : 0;
  if (win_b) *win_b = units * (size_t)W_cap * kD * 2;
  return KVMIX_OK;
}

int kvmix_workspace_bytes(const kvmix_shape* sh, int T_max, size_t* bytes) {
  kvmix_layer_cfg cfg = {2, 2, 0};
  const int st = check_shape_cfg(sh, &cfg);
  if (st) return st;
  if (!bytes) return KVMIX_ERR_NULL;
  if (T_max < 0) return KVMIX_ERR_BAD_SHAPE;
  const size_t units = (size_t)sh->B * sh->Hkv, G = (size_t)(sh->Hq / sh->Hkv);
  *bytes = counters_bytes(out_units(sh)) + units * (size_t)(max_splits(sh) + 1) * G * (kD + 2) * sizeof(float);
  return KVMIX_OK;
}

int kvmix_quantize_pack(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* k_fp16, const uint16_t* v_fp16,
                        int64_t token_stride, int64_t head_stride, int64_t batch_stride, int n_tokens, int t0,
                        const kvmix_layer_cache* c, void* stream) {
  int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (cfg->k_bits == 16) return KVMIX_ERR_BAD_BITS;
  if (!k_fp16 || !v_fp16) return KVMIX_ERR_NULL;
  st = check_cache(cfg, c, true);
  if (st) return st;
  if (n_tokens < 0 || n_tokens % kTile || t0 < 0 || t0 % kTile || (long long)t0 + n_tokens > c->T_cap) return KVMIX_ERR_BAD_SHAPE;
  if (!aligned16(k_fp16) || !aligned16(v_fp16) || token_stride % 8 || head_stride % 8 || batch_stride % 8 || token_stride < kD)
    return KVMIX_ERR_ALIGN;
  QuantArgs a{};
  a.k = k_fp16; a.v = v_fp16;
  a.k_tok = token_stride; a.k_unit_b = batch_stride; a.k_unit_h = head_stride;
  a.v_tok = token_stride; a.v_unit_b = batch_stride; a.v_unit_h = head_stride;
  a.n_ring = 0; a.W_cap = 1;
  fill_quant_dst(a, c);
  a.tile0 = t0 / kTile;
  a.Hkv = sh->Hkv;
  const hipError_t e = launch_quantize_pack(a, cfg->k_bits, cfg->v_bits, n_tokens / kTile, sh->B * sh->Hkv, (hipStream_t)stream);
  return e == hipSuccess ? KVMIX_OK : hip_fail(e);
}

int kvmix_append_tokens(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* k_new, const uint16_t* v_new,
                        int64_t token_stride, int64_t head_stride, int64_t batch_stride, int n_tokens,
                        kvmix_layer_cache* c, void* stream) {
  int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (!k_new || !v_new) return KVMIX_ERR_NULL;
  const bool packed = cfg->k_bits != 16;
  st = check_cache(cfg, c, packed);
  if (st) return st;
  if (n_tokens < 0) return KVMIX_ERR_BAD_SHAPE;
  if (token_stride < kD || head_stride < 0 || batch_stride < 0) return KVMIX_ERR_ALIGN;
  if (packed && (!aligned16(k_new) || !aligned16(v_new) || token_stride % 8 || head_stride % 8 || batch_stride % 8)) return KVMIX_ERR_ALIGN;
  const bool ageing = packed && cfg->window >= 0;    // this call flushes; otherwise it only fills the ring
  if (ageing && c->v_lead != 0) return KVMIX_ERR_BAD_SHAPE;
  if (ageing && c->W_cap < cfg->window + kTile) return KVMIX_ERR_BAD_SHAPE;
  // dry run of the counters: nothing is launched unless everything fits
  {
    long long n_q = c->n_q, n_w = c->n_w;
    if (ring_tokens(c) >= c->W_cap && n_tokens > 0) return KVMIX_ERR_BAD_SHAPE;
    if (!ageing) {
      if ((long long)ring_tokens(c) + n_tokens > c->W_cap) return KVMIX_ERR_BAD_SHAPE;
    } else {
      if (n_w >= cfg->window + kTile && n_tokens > 0) return KVMIX_ERR_BAD_SHAPE;   // a flush is overdue: not a state this library leaves
      const long long flushes = (n_w + n_tokens) >= cfg->window + kTile ? (n_w + n_tokens - cfg->window) / kTile : 0;
      if (n_q + flushes * kTile > c->T_cap) return KVMIX_ERR_BAD_SHAPE;
    }
  }
  if (n_tokens == 0) return KVMIX_OK;
  const int units = sh->B * sh->Hkv, W = c->W_cap;
  // The old window tokens followed by the new ones form one sequence of m rows; its first 32 F rows leave for the
  // packed part (F tiles, from the ring or straight from the input: a token that is flushed within this call never
  // passes through the ring), the rest is the new window. Two launches: the quantizer over the F tiles, then the copy
  // of the surviving new rows into their ring slots (in this order: a new row may land in the slot of an old one
  // that the quantizer still has to read).
  const long long m = (long long)c->n_w + n_tokens;
  const int F = ageing && m >= cfg->window + kTile ? (int)((m - cfg->window) / kTile) : 0;
  if (F > 0) {
    QuantArgs a{};
    a.k = k_new; a.v = v_new;
    a.k_tok = token_stride; a.k_unit_b = batch_stride; a.k_unit_h = head_stride;
    a.v_tok = token_stride; a.v_unit_b = batch_stride; a.v_unit_h = head_stride;
    a.k_ring = c->k_win; a.v_ring = c->v_win; a.n_ring = c->n_w; a.ring_w0 = c->w0; a.W_cap = W;
    fill_quant_dst(a, c);
    a.tile0 = c->n_q / kTile;
    a.Hkv = sh->Hkv;
    const hipError_t e = launch_quantize_pack(a, cfg->k_bits, cfg->v_bits, F, units, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
  }
  const long long first_kept = (long long)F * kTile;                       // first row of the sequence that stays in the window
  const int i0 = first_kept > c->n_w ? (int)(first_kept - c->n_w) : 0;      // first new token that stays
  if (i0 < n_tokens) {
    AppendArgs ap{};
    ap.k_new = k_new + (int64_t)i0 * token_stride; ap.v_new = v_new + (int64_t)i0 * token_stride;
    ap.tok = token_stride; ap.head = head_stride; ap.batch = batch_stride;
    ap.k_win = c->k_win; ap.v_win = c->v_win;
    ap.W_cap = W; ap.slot = (int)((c->w0 + c->n_w + (long long)i0) % W); ap.n = n_tokens - i0; ap.units = units; ap.Hkv = sh->Hkv;
    const hipError_t e = launch_append(ap, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
  }
  c->n_q += F * kTile;
  c->w0 = (int)((c->w0 + first_kept) % W);
  c->n_w = (int)(m - first_kept);
  return KVMIX_OK;
}

int kvmix_append(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* k_new, const uint16_t* v_new,
                 kvmix_layer_cache* c, void* stream) {
  if (!sh) return KVMIX_ERR_NULL;
  return kvmix_append_tokens(sh, cfg, k_new, v_new, kD, kD, (int64_t)sh->Hkv * kD, 1, c, stream);
}

}  // extern "C"

namespace {

// Everything an attention launch needs, filled by plan_attention after all host-side checks have passed.
// `mixed`: the fronts of Keys and Values differ; the tokens between them go to a launch of their own (m) that
// leaves one more partial for the main launch's merge.
struct AttnPlan { AttnArgs a; int kb, vb, G, units; bool mixed; MixedArgs m; };

size_t split_workspace_bytes(int units, int n_parts, int G) {
  return counters_bytes(units * (G > 8 ? G / 8 : 1)) + (size_t)units * n_parts * G * (kD + 2) * sizeof(float);
}

// How an attention call divides the n = n_q + n_w tokens of a cache whose Value front is n_q + v_lead:
// tiles [0, packed_tiles) have Keys and Values packed, tokens [32 packed_tiles, t_a) are the mixed range, tokens
// [t_a, n) are window tokens of both (t_a is a multiple of 32 unless it equals n).
struct Fronts { int packed_tiles; long long t_a; int n_w_eff, w0_eff; bool mixed; };
Fronts fronts_of(const kvmix_layer_cache* c, int n_w) {
  Fronts f;
  const long long n = (long long)c->n_q + n_w, n_qv = (long long)c->n_q + c->v_lead;
  if (c->v_lead == 0) {
    f.packed_tiles = c->n_q / kTile; f.t_a = c->n_q; f.n_w_eff = n_w; f.w0_eff = c->w0; f.mixed = false;
    return f;
  }
  const long long lo = n_qv < c->n_q ? n_qv : c->n_q, hi = n_qv < c->n_q ? c->n_q : n_qv;
  f.packed_tiles = (int)(lo / kTile);
  long long t_a = (hi + kTile - 1) / kTile * kTile;
  if (t_a > n) t_a = n;
  f.t_a = t_a;
  f.n_w_eff = (int)(n - t_a);
  f.w0_eff = f.n_w_eff > 0 ? slot_of(c, t_a) : 0;
  f.mixed = true;
  return f;
}

// Validates an attention call against the cache state `c` (window count n_w) and fills the launch descriptor;
// launches nothing. With k_new / v_new the newest token of every unit is taken from there (ring slot new_slot,
// counted in n_w) and stored into the window by the kernel.
int plan_attention(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* q, const kvmix_layer_cache* c, int n_w,
                   const uint16_t* k_new, const uint16_t* v_new, int new_slot,
                   float softmax_scale, uint16_t* out, void* workspace, size_t workspace_bytes, int n_splits, AttnPlan* plan) {
  int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (!q || !out) return KVMIX_ERR_NULL;
  if (!aligned16(q) || !aligned16(out)) return KVMIX_ERR_ALIGN;
  st = check_cache(cfg, c, false);
  if (st) return st;
  if (c->n_q + n_w < 1 || n_w < 0 || n_w > c->W_cap || (long long)n_w - (c->v_lead < 0 ? c->v_lead : 0) > c->W_cap) return KVMIX_ERR_BAD_SHAPE;
  const int units = sh->B * sh->Hkv, G = sh->Hq / sh->Hkv;
  const Fronts fr = fronts_of(c, n_w);
  const int n_items = c->W_cap / kTile + fr.packed_tiles;
  if (n_splits < 0 || n_splits > max_splits(sh)) return KVMIX_ERR_BAD_SHAPE;
  if (n_splits == 0) {
    // One workgroup occupies a whole compute unit (LDS), so the launch runs in rounds of `cus` workgroups. A round
    // costs a fixed part (start, merge of the waves, partial and arrival: about what 48 tiles take) plus the tiles
    // of one split; take the split count with the smallest rounds x (48 + tiles per split), at least 8 tiles each.
    const int cus = num_cus();
    if (cus == 0) return hip_fail(hipErrorInvalidDevice);
    const int ou = out_units(sh);
    int s_max = n_items / 8;
    if (s_max > max_splits(sh)) s_max = max_splits(sh);
    double best = 0.0, unsplit = 0.0;
    n_splits = 1;
    for (int s = 1; s <= s_max || s == 1; s++) {
      const double rounds = (double)(((long long)ou * s + cus - 1) / cus);
      const double cost = rounds * (48.0 + (double)n_items / s);
      if (s == 1) unsplit = cost;
      if (s == 1 || cost < best) { best = cost; n_splits = s; }
    }
    // an unsplit launch has no partials to write and merge, which the model leaves out: it wins a near tie
    // (multi-query shape with 288 workgroups: 51 us unsplit, 55 us with 2 splits, modelled 352 against 336)
    if (unsplit <= 1.06 * best) n_splits = 1;
  }
  if (n_splits > n_items) n_splits = n_items;
  AttnArgs a{};
  const int n_parts = n_splits + (fr.mixed ? 1 : 0);
  if (n_parts > 1) {
    if (!workspace) return KVMIX_ERR_NULL;
    if (!aligned16(workspace)) return KVMIX_ERR_ALIGN;
    if (workspace_bytes < split_workspace_bytes(units, n_parts, G)) return KVMIX_ERR_WORKSPACE;
    a.counters = reinterpret_cast<uint32_t*>(workspace);
    a.part = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + counters_bytes(out_units(sh)));
  }
  a.q = q; a.out = out;
  a.packed = c->packed;
  a.k_win = c->k_win; a.v_win = c->v_win;
  a.k_new = k_new; a.v_new = v_new; a.k_win_w = c->k_win; a.v_win_w = c->v_win; a.new_slot = new_slot;
  a.tiles_cap = c->T_cap / kTile; a.W_cap = c->W_cap; a.n_tiles = fr.packed_tiles; a.n_w = fr.n_w_eff; a.w0 = fr.w0_eff;
  a.Hq = sh->Hq; a.Hkv = sh->Hkv; a.n_splits = n_splits; a.n_parts = n_parts;
  a.items_q = n_items / n_splits; a.items_r = n_items % n_splits;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)kD);
  a.scale_log2 = scale * 1.4426950408889634f;
  plan->a = a;
  plan->kb = cfg->k_bits == 16 ? 2 : cfg->k_bits;
  plan->vb = cfg->v_bits == 16 ? 2 : cfg->v_bits;
  plan->G = G; plan->units = units;
  plan->mixed = fr.mixed;
  if (fr.mixed) {
    // with the append inside the launch the new token must be a window token of the main launch
    if (new_slot >= 0 && fr.n_w_eff < 1) return KVMIX_ERR_BAD_SHAPE;
    MixedArgs m{};
    m.q = q; m.packed = c->packed; m.k_win = c->k_win; m.v_win = c->v_win;
    m.part = a.part; m.n_parts = n_parts; m.part_index = n_splits;
    m.tiles_cap = a.tiles_cap; m.W_cap = c->W_cap; m.k_bits = plan->kb; m.v_bits = plan->vb;
    m.n_qk = c->n_q; m.n_qv = c->n_q + c->v_lead;
    m.t_begin = fr.packed_tiles * kTile; m.t_end = (int)fr.t_a;
    m.slot_begin = slot_of(c, m.t_begin);
    m.G = G; m.G_main = G > 8 ? 8 : G;
    m.scale_log2 = a.scale_log2;
    plan->m = m;
  }
  return KVMIX_OK;
}

int launch_plan(const AttnPlan& p, void* stream) {
  if (p.mixed) {
    const hipError_t e = launch_mixed_fronts(p.m, p.units, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
  }
  const hipError_t e = launch_decode_attn(p.a, p.kb, p.vb, p.G, p.units, (hipStream_t)stream);
  return e == hipSuccess ? KVMIX_OK : hip_fail(e);
}

// ---- split workspace of kvmix_decode_attn_static: a fixed array in device memory, one copy per GPU
constexpr size_t kScratchBytes = KVMIX_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
// In host code the array's name is only a handle; its address on a device comes from hipGetSymbolAddress,
// asked once per device with that device current. Each GPU holds its own copy at its own address.
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

__global__ void clear_words_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Address of the current device's copy of `scratch`. The first call on a device also clears the array (the
// arrival counters sit at its start) on `stream`, ahead of the first launch that uses it; afterwards every
// attention launch leaves the counters zero again.
int scratch_address(void** ptr, hipStream_t stream) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!p) return hip_fail(hipErrorInvalidSymbol);
    constexpr int kWords = (int)(kScratchBytes / 4);       // the whole array: the counters sit at its start, however many
    clear_words_kernel<<<kWords / 256, 256, 0, stream>>>(reinterpret_cast<uint32_t*>(p), kWords);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return KVMIX_OK;
}

}  // namespace

extern "C" {

int kvmix_decode_attn(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* q, const kvmix_layer_cache* c,
                      float softmax_scale, uint16_t* out, void* workspace, size_t workspace_bytes, int n_splits, void* stream) {
  const int st0 = check_shape_cfg(sh, cfg);   // before the cache struct is looked at
  if (st0) return st0;
  if (!q || !out) return KVMIX_ERR_NULL;
  if (!aligned16(q) || !aligned16(out)) return KVMIX_ERR_ALIGN;
  if (!c) return KVMIX_ERR_NULL;
  AttnPlan plan;
  const int st = plan_attention(sh, cfg, q, c, c->n_w, nullptr, nullptr, -1, softmax_scale, out, workspace, workspace_bytes, n_splits, &plan);
  return st ? st : launch_plan(plan, stream);
}

int kvmix_decode_attn_static(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* q, const kvmix_layer_cache* c,
                             float softmax_scale, uint16_t* out, int n_splits, void* stream) {
  const int st0 = check_shape_cfg(sh, cfg);
  if (st0) return st0;
  if (!q || !out) return KVMIX_ERR_NULL;
  if (!aligned16(q) || !aligned16(out)) return KVMIX_ERR_ALIGN;
  if (!c) return KVMIX_ERR_NULL;
  AttnPlan plan;
  // First pass with a workspace of "any size" at a dummy aligned address: settles the split count and runs
  // every other check; the size that split count needs is then held against the array's fixed size.
  int st = plan_attention(sh, cfg, q, c, c->n_w, nullptr, nullptr, -1, softmax_scale, out, reinterpret_cast<void*>(256), ~(size_t)0, n_splits, &plan);
  if (st) return st;
  if (plan.a.n_parts > 1) {
    if (split_workspace_bytes(plan.units, plan.a.n_parts, plan.G) > kScratchBytes) return KVMIX_ERR_WORKSPACE;
    void* ptr = nullptr;
    st = scratch_address(&ptr, (hipStream_t)stream);
    if (st) return st;
    plan.a.counters = reinterpret_cast<uint32_t*>(ptr);
    plan.a.part = reinterpret_cast<float*>(reinterpret_cast<char*>(ptr) + counters_bytes(plan.units * (plan.G > 8 ? plan.G / 8 : 1)));
    plan.m.part = plan.a.part;
  } else {
    plan.a.counters = nullptr; plan.a.part = nullptr;
  }
  return launch_plan(plan, stream);
}

int kvmix_decode_step(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const uint16_t* k_new, const uint16_t* v_new,
                      const uint16_t* q, kvmix_layer_cache* c, float softmax_scale, uint16_t* out,
                      void* workspace, size_t workspace_bytes, int n_splits, void* stream) {
  int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (!k_new || !v_new || !c) return KVMIX_ERR_NULL;
  AttnPlan plan;
  const bool flush = cfg->k_bits != 16 && cfg->window >= 0 && c->n_w + 1 == cfg->window + kTile;
  if (cfg->k_bits != 16 && cfg->window >= 0 && c->v_lead != 0) return KVMIX_ERR_BAD_SHAPE;   // fixed-window ageing needs one front
  if (flush) {
    // The 32 oldest window tokens move to the packed part before the attention reads them. Every check is made
    // first, the attention's against the counters as the flush will leave them, so that a failing call launches
    // nothing and leaves the counters alone.
    st = check_cache(cfg, c, true);
    if (st) return st;
    if (c->n_q + kTile > c->T_cap || c->W_cap < cfg->window + kTile) return KVMIX_ERR_BAD_SHAPE;
    if (!aligned16(k_new) || !aligned16(v_new)) return KVMIX_ERR_ALIGN;
    kvmix_layer_cache after = *c;
    after.n_q += kTile; after.n_w = c->n_w + 1 - kTile; after.w0 = (c->w0 + kTile) % c->W_cap;
    if (cfg->window >= kTile) {
      // The new token is not among the 32 oldest: quantize-and-pack them straight from the ring (one launch), then
      // the attention launch with the append inside, as on every other step.
      const int slot = (c->w0 + c->n_w) % c->W_cap;
      st = plan_attention(sh, cfg, q, &after, after.n_w, k_new, v_new, slot, softmax_scale, out, workspace, workspace_bytes, n_splits, &plan);
      if (st) return st;
      const int W = c->W_cap;
      QuantArgs qa{};
      qa.k_ring = c->k_win; qa.v_ring = c->v_win; qa.n_ring = kTile; qa.ring_w0 = c->w0; qa.W_cap = W;
      fill_quant_dst(qa, c);
      qa.tile0 = c->n_q / kTile;
      qa.Hkv = sh->Hkv;
      const hipError_t e = launch_quantize_pack(qa, cfg->k_bits, cfg->v_bits, 1, sh->B * sh->Hkv, (hipStream_t)stream);
      if (e != hipSuccess) return hip_fail(e);
      c->n_q = after.n_q; c->w0 = after.w0; c->n_w = after.n_w - 1;   // the flush is done; the append follows
      st = launch_plan(plan, stream);
      if (st) return st;
      c->n_w += 1;
      return KVMIX_OK;
    }
    // window length 0: the new token is itself among the 32 that are flushed; append, quantize-pack, attention
    st = plan_attention(sh, cfg, q, &after, after.n_w, nullptr, nullptr, -1, softmax_scale, out, workspace, workspace_bytes, n_splits, &plan);
    if (st) return st;
    st = kvmix_append(sh, cfg, k_new, v_new, c, stream);
    if (st) return st;
    return launch_plan(plan, stream);
  }
  st = check_cache(cfg, c, cfg->k_bits != 16);
  if (st) return st;
  if (ring_tokens(c) >= c->W_cap) return KVMIX_ERR_BAD_SHAPE;
  if (cfg->k_bits != 16 && c->W_cap < cfg->window + kTile) return KVMIX_ERR_BAD_SHAPE;
  if (!aligned16(k_new) || !aligned16(v_new)) return KVMIX_ERR_ALIGN;
  if (c->v_lead != 0 && fronts_of(c, c->n_w + 1).t_a > (long long)c->n_q + c->n_w) {
    // The new token shares its tile with the younger front: it belongs to the range between the fronts, which is
    // read from the ring by a launch of its own. Plan against the counters as the append will leave them, append,
    // then the two attention launches.
    kvmix_layer_cache after = *c;
    after.n_w += 1;
    st = plan_attention(sh, cfg, q, &after, after.n_w, nullptr, nullptr, -1, softmax_scale, out, workspace, workspace_bytes, n_splits, &plan);
    if (st) return st;
    st = kvmix_append(sh, cfg, k_new, v_new, c, stream);
    if (st) return st;
    return launch_plan(plan, stream);
  }
  const int slot = (c->w0 + c->n_w) % c->W_cap;
  // the kernel's window count includes the new token: it is read from k_new / v_new in place of its ring row (and stored)
  st = plan_attention(sh, cfg, q, c, c->n_w + 1, k_new, v_new, slot, softmax_scale, out, workspace, workspace_bytes, n_splits, &plan);
  if (st) return st;
  st = launch_plan(plan, stream);
  if (st) return st;
  c->n_w += 1;
  return KVMIX_OK;
}

int kvmix_rpc_next(double r_k, double r_v, int current_k, int current_v, int* num_k, int* num_v) {
  if (!num_k || !num_v) return KVMIX_ERR_NULL;
  if (!(r_k >= 0.0 && r_k <= 1.0) || !(r_v >= 0.0 && r_v <= 1.0) || current_k < 0 || current_v < 0) return KVMIX_ERR_BAD_SHAPE;
  *num_k = (int)std::floor(r_k * (double)current_k);
  *num_v = (int)std::floor(r_v * (double)current_v);
  return KVMIX_OK;
}

int kvmix_flush(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, kvmix_layer_cache* c, int keep_k, int keep_v, void* stream) {
  int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (cfg->k_bits == 16) return KVMIX_ERR_BAD_BITS;
  st = check_cache(cfg, c, true);
  if (st) return st;
  if (keep_k < 0 || keep_v < 0) return KVMIX_ERR_BAD_SHAPE;
  const long long n = (long long)c->n_q + c->n_w, n_qv = (long long)c->n_q + c->v_lead;
  long long nk = n - keep_k, nv = n - keep_v;
  if (nk < 0) nk = 0;
  nk -= nk % kTile;
  if (nk < c->n_q) nk = c->n_q;
  if (nv < n_qv) nv = n_qv;
  if (nk > c->T_cap || nv > c->T_cap) return KVMIX_ERR_BAD_SHAPE;
  const bool k_moves = nk > c->n_q, v_moves = nv > n_qv;
  if (!k_moves && !v_moves) return KVMIX_OK;
  // one launch over the tiles that either side touches
  long long first = k_moves ? c->n_q / kTile : n_qv / kTile, last = k_moves ? nk / kTile : (nv + kTile - 1) / kTile;
  if (v_moves) {
    if (n_qv / kTile < first) first = n_qv / kTile;
    if ((nv + kTile - 1) / kTile > last) last = (nv + kTile - 1) / kTile;
  }
  QuantArgs a{};
  a.k_ring = c->k_win; a.v_ring = c->v_win; a.W_cap = c->W_cap;
  a.ring_w0 = slot_of(c, first * kTile);
  fill_quant_dst(a, c);
  a.tile0 = (int)first;
  a.Hkv = sh->Hkv;
  a.k_tile_a = c->n_q / kTile; a.k_tile_b = (int)(nk / kTile);
  a.v_tok_a = (int)n_qv; a.v_tok_b = (int)nv;
  const hipError_t e = launch_quantize_fronts(a, cfg->k_bits, cfg->v_bits, (int)(last - first), sh->B * sh->Hkv, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  c->w0 = slot_of(c, nk);
  c->n_q = (int)nk;
  c->n_w = (int)(n - nk);
  c->v_lead = (int)(nv - nk);
  return KVMIX_OK;
}

int kvmix_stream_read(const void* buf, size_t bytes, int workgroups, int threads, void* sink, void* stream) {
  if (!buf) return KVMIX_ERR_NULL;
  if (!aligned16(buf)) return KVMIX_ERR_ALIGN;
  if (workgroups < 1 || workgroups > 65535 || threads < 64 || threads > 768 || threads % 64) return KVMIX_ERR_BAD_SHAPE;
  const hipError_t e = launch_stream_read(buf, bytes, workgroups, threads, reinterpret_cast<uint32_t*>(sink), (hipStream_t)stream);
  return e == hipSuccess ? KVMIX_OK : hip_fail(e);
}

int kvmix_dequant(const kvmix_shape* sh, const kvmix_layer_cfg* cfg, const kvmix_layer_cache* c, int which, float* out, void* stream) {
  int st = check_shape_cfg(sh, cfg);
  if (st) return st;
  if (cfg->k_bits == 16) return KVMIX_ERR_BAD_BITS;
  if (!out) return KVMIX_ERR_NULL;
  if (which != 0 && which != 1) return KVMIX_ERR_BAD_SHAPE;
  st = check_cache(cfg, c, true);
  if (st) return st;
  DequantArgs a{};
  a.packed = c->packed;
  a.out = out; a.tiles_cap = c->T_cap / kTile; a.n_tokens = c->n_q + (which ? c->v_lead : 0);
  a.k_bits = cfg->k_bits; a.v_bits = cfg->v_bits; a.which = which;
  const hipError_t e = launch_dequant(a, sh->B * sh->Hkv, (hipStream_t)stream);
  return e == hipSuccess ? KVMIX_OK : hip_fail(e);
}

}  // extern "C"
