// C ABI of the hybrid-attention library: host-side validation, workspace planning and the launch
// sequence.  Nothing here touches the device except through the launchers and hipMemcpyAsync.
#include <cmath>
#include <cstring>
#include <mutex>

#include "ha_plan.h"

namespace ha {

static thread_local int g_last_device_error = 0;

// Optional per-stage event records (benchmark tap): 6 events per record.
struct Profile {
  hipEvent_t *ev = nullptr;
  int n = 0, count = 0;
  bool dominant_only = false;   // record only the pair around the dominant kernel (two events per forward)
};
static thread_local Profile g_prof;
static inline hipEvent_t *prof_events() {
  return g_prof.n > 0 ? g_prof.ev + (size_t)(g_prof.count % g_prof.n) * 6 : nullptr;
}

static inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }
static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static ha_status check_map(const ha_feature_map *fm, const ha_problem &p) {
  if (!fm->w1 || !fm->w2) return HA_ERR_NULL;
  if (fm->d_hidden <= 0 || fm->d_out <= 0 || fm->poly_degree < 1) return HA_ERR_SHAPE;
  if (fm->d_out % fm->poly_degree != 0) return HA_ERR_SHAPE;
  if (fm->poly_degree > 8) return HA_ERR_UNSUPPORTED;
  if (fm->out_act != HA_ACT_SOFTMAX && fm->out_act != HA_ACT_EXP && fm->out_act != HA_ACT_RELU) return HA_ERR_UNSUPPORTED;
  const bool square = fm->d_hidden == p.d_head && fm->d_out == p.d_head;
  const bool paper_width = p.d_head == 128 && fm->d_hidden == 256 && fm->d_out == 256;
  // any other width goes layer by layer through HBM (ha_wide.hip): multiples of 128 up to 768 (Tab. "phi": P d, P <= 6)
  const bool layered = p.d_head == 128 && fm->d_hidden % 128 == 0 && fm->d_out % 128 == 0 && fm->d_hidden <= 768 &&
                       fm->d_out <= 768;
  if (fm->w_mid) {   // three layers: always layer by layer
    if (fm->d_mid <= 0) return HA_ERR_SHAPE;
    if (!layered || fm->d_mid % 128 != 0 || fm->d_mid > 768) return HA_ERR_UNSUPPORTED;
    if (!aligned16(fm->w_mid) || (fm->b_mid && (reinterpret_cast<uintptr_t>(fm->b_mid) & 3u))) return HA_ERR_ALIGN;
  }
  if (!square && !paper_width && !layered) return HA_ERR_UNSUPPORTED;
  if (!aligned16(fm->w1) || !aligned16(fm->w2)) return HA_ERR_ALIGN;
  if ((fm->b1 && (reinterpret_cast<uintptr_t>(fm->b1) & 3u)) || (fm->b2 && (reinterpret_cast<uintptr_t>(fm->b2) & 3u)))
    return HA_ERR_ALIGN;
  return HA_OK;
}

static ha_status validate(const ha_problem *p, const ha_feature_map *phi_q, const ha_feature_map *phi_k) {
  if (!p) return HA_ERR_NULL;
  if (p->B <= 0 || p->H <= 0 || p->N <= 0 || p->d_head <= 0) return HA_ERR_SHAPE;
  if (p->hybrid_rate < 0 || p->hybrid_rate > p->N) return HA_ERR_SHAPE;
  if (p->split_granularity < 0 || p->split_granularity > p->N || p->causal_chunk < 0) return HA_ERR_SHAPE;
  if ((int64_t)p->hybrid_rate * p->split_granularity > (int64_t)1 << 30) return HA_ERR_UNSUPPORTED;
  if (!(p->softmax_scale > 0.f) || !std::isfinite(p->softmax_scale)) return HA_ERR_SHAPE;
  if (p->dtype != HA_BF16 && p->dtype != HA_F32) return HA_ERR_UNSUPPORTED;
  if (p->d_head != 64 && p->d_head != 128) return HA_ERR_UNSUPPORTED;
  if (p->block_size != 64 && p->block_size != 128) return HA_ERR_UNSUPPORTED;
  if (p->stride_n < p->d_head || p->stride_h <= 0 || p->stride_b <= 0) return HA_ERR_SHAPE;
  if ((int64_t)p->B * p->H > 65535) return HA_ERR_UNSUPPORTED;
  const int per16 = p->dtype == HA_BF16 ? 8 : 4;   // elements per 16 bytes
  if (p->stride_n % per16 || p->stride_h % per16 || p->stride_b % per16) return HA_ERR_ALIGN;
  const bool has_linear = p->hybrid_rate != 1;
  if (has_linear) {
    if (!phi_q || !phi_k) return HA_ERR_NULL;
    ha_status s = check_map(phi_q, *p);
    if (s != HA_OK) return s;
    s = check_map(phi_k, *p);
    if (s != HA_OK) return s;
    if (phi_q->d_out != phi_k->d_out || phi_q->d_hidden != phi_k->d_hidden) return HA_ERR_SHAPE;
    if (phi_q->poly_degree != phi_k->poly_degree) return HA_ERR_SHAPE;
    if ((phi_q->w_mid != nullptr) != (phi_k->w_mid != nullptr)) return HA_ERR_SHAPE;
    if (phi_q->w_mid && phi_q->d_mid != phi_k->d_mid) return HA_ERR_SHAPE;
  }
  if (p->local_window < 0 || p->reserved != 0) return HA_ERR_SHAPE;
  if (p->local_window > 0) {
    if (p->hybrid_rate != 0 || p->split_granularity > 1 || p->causal_chunk != 0) return HA_ERR_SHAPE;
    if (p->local_window % (2 * p->block_size)) return HA_ERR_UNSUPPORTED;      // whole query tiles
  }
  if (p->causal_chunk > 0 || p->local_window > 0) {
    if (p->causal_chunk % (2 * p->block_size)) return HA_ERR_UNSUPPORTED;      // whole query tiles per chunk
    if (has_linear) {
      const bool square = phi_q->d_hidden == p->d_head && phi_q->d_out == p->d_head;
      const bool paper_width = p->d_head == 128 && phi_q->d_hidden == 256 && phi_q->d_out == 256;
      if ((!square && !paper_width) || phi_q->w_mid) return HA_ERR_UNSUPPORTED;   // the layer-by-layer path has no prefix states
    }
  }
  return HA_OK;
}

void make_plan(const ha_problem &p, const ha_feature_map *phi_q, const ha_feature_map *phi_k, Plan &pl) {
  std::memset(&pl, 0, sizeof(pl));
  pl.B = p.B; pl.H = p.H; pl.N = p.N; pl.D = p.d_head; pl.R = p.hybrid_rate;
  pl.f32 = p.dtype == HA_F32;
  pl.sb = p.stride_b; pl.sh = p.stride_h; pl.sn = p.stride_n;
  pl.scale = p.softmax_scale;
  pl.G = p.split_granularity > 1 ? p.split_granularity : 1;
  // softmax tokens: the first G of every R G tokens
  pl.NS = pl.R == 0 ? 0 : (pl.N / (pl.R * pl.G)) * pl.G + (pl.N % (pl.R * pl.G) < pl.G ? pl.N % (pl.R * pl.G) : pl.G);
  pl.CC = p.causal_chunk < p.N ? p.causal_chunk : 0;      // one chunk that covers everything is the plain operator
  pl.n_cc = pl.CC > 0 ? (pl.N + pl.CC - 1) / pl.CC : 1;
  pl.nsub = 1;
  pl.LW = p.local_window;
  if (pl.LW > 0) {
    // every token is a candidate softmax key (compacted at rate 1) and a linear key of the tiles that do not see it
    pl.NS = pl.N;
    pl.CC = 2 * p.block_size;                             // one state-pass chunk and one state per query tile
    pl.n_cc = (pl.N + pl.CC - 1) / pl.CC;
  }
  pl.NL = pl.LW > 0 ? pl.N : pl.N - pl.NS;
  const bool has_linear = pl.NL > 0 && phi_q && phi_k;
  pl.HD = has_linear ? phi_k->d_hidden : pl.D;
  pl.F = has_linear ? phi_k->d_out : pl.D;
  pl.P = has_linear ? phi_k->poly_degree : 1;
  pl.DM = has_linear && phi_k->w_mid ? phi_k->d_mid : 0;
  pl.act_q = has_linear ? phi_q->out_act : 0;
  pl.act_k = has_linear ? phi_k->out_act : 0;
  pl.KT = p.block_size;
  pl.QT = 2 * p.block_size;
  pl.n_qtiles = (pl.N + pl.QT - 1) / pl.QT;
  pl.n_ktiles = (pl.NS + pl.KT - 1) / pl.KT;
  pl.n_kblocks = pl.n_ktiles * (pl.KT / 32);
  // state pass: one workgroup per CU (256 CUs) in a single round when there is enough work,
  // chunks are whole 128-token tiles
  {
    const int tiles = (pl.NL + 127) / 128;
    const int per_head = 256 / (pl.B * pl.H) > 0 ? 256 / (pl.B * pl.H) : 1;
    const int want = tiles < per_head ? (tiles > 0 ? tiles : 1) : per_head;
    pl.CH = ((tiles + want - 1) / want) * 128;
    if (pl.CH < 128) pl.CH = 128;
    pl.n_chunks = has_linear ? (pl.NL + pl.CH - 1) / pl.CH : 0;
    if (pl.LW > 0) {
      pl.CH = pl.CC;
      pl.n_chunks = pl.n_cc;
    } else if (pl.CC > 0 && has_linear) {
      // chunk-causal: every causal chunk is a group of nsub state-pass workgroups of its own; CH from the most linear
      // tokens a chunk can hold
      int most = 0;
      for (int c = 0; c < pl.n_cc; ++c) {
        const int lo = c * pl.CC, hi = (c + 1) * pl.CC < pl.N ? (c + 1) * pl.CC : pl.N;
        const int cnt = (hi - lo) - (softmax_before(hi, pl.R, pl.G) - softmax_before(lo, pl.R, pl.G));
        most = cnt > most ? cnt : most;
      }
      const int tiles_c = (most + 127) / 128 > 0 ? (most + 127) / 128 : 1;
      const int room = 256 / (pl.B * pl.H * pl.n_cc);
      pl.nsub = room < 1 ? 1 : (room > tiles_c ? tiles_c : room);
      pl.CH = ((tiles_c + pl.nsub - 1) / pl.nsub) * 128;
      pl.n_chunks = pl.n_cc * pl.nsub;
    }
  }
  pl.n_state_tiles = (pl.F / 32) * (pl.D / 32 + 1);
  const size_t BH = (size_t)pl.B * pl.H;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  pl.off_w1q = take((size_t)pl.H * pl.HD * pl.D * 2);
  pl.off_w2q = take((size_t)pl.H * pl.F * pl.HD * 2);
  pl.off_w1k = take((size_t)pl.H * pl.HD * pl.D * 2);
  pl.off_w2k = take((size_t)pl.H * pl.F * pl.HD * 2);
  pl.off_ks = take(BH * pl.n_kblocks * 32 * pl.D * 2);
  pl.off_vs = take(BH * pl.n_kblocks * 32 * pl.D * 2);
  pl.off_part = take(BH * pl.n_chunks * pl.n_state_tiles * 1024 * 4);
  pl.off_S = take(BH * pl.F * pl.D * 4);
  pl.off_z = take(BH * pl.n_cc * pl.F * 4);
  pl.off_sthi = take(BH * pl.n_cc * pl.F * pl.D * 2);
  pl.off_stlo = take(BH * pl.n_cc * pl.F * pl.D * 2);
  pl.total = off;
}

// Feature maps outside the fused kernels' widths take the layer-by-layer path.
static bool needs_wide_path(const Plan &pl) {
  const bool square = pl.HD == pl.D && pl.F == pl.D;
  const bool paper_width = pl.D == 128 && pl.HD == 256 && pl.F == 256;
  return pl.NL > 0 && ((!square && !paper_width) || pl.DM > 0);
}

// Plan of the forward plus, where needed, the layer-by-layer path's buffers behind it; returns the workspace size.
static size_t full_plan(const ha_problem &p, const ha_feature_map *phi_q, const ha_feature_map *phi_k, Plan &pl, WidePlan &wp,
                        bool &wide) {
  make_plan(p, phi_q, phi_k, pl);
  wide = phi_q && phi_k && needs_wide_path(pl);
  if (!wide) return pl.total;
  make_wide_plan(pl, pl.total, wp);
  return wp.total;
}

static ha_status device_error(hipError_t e) {
  g_last_device_error = static_cast<int>(e);
  return HA_ERR_DEVICE;
}

// ev (optional): ev[0] before compaction, ev[1] after it, ev[2] after the state is reduced.
// prep_q (optional): the query-side map; where the plain reduction runs, its weights are re-ordered in the same launch
// and *prep_q_done is set.
static ha_status run_key_side(const Plan &pl, const void *k, const void *v, const ha_feature_map *phi_k, void *ws,
                              hipStream_t st, hipEvent_t *ev = nullptr, const WidePlan *wide = nullptr,
                              const ha_feature_map *prep_q = nullptr, bool *prep_q_done = nullptr) {
  hipError_t e;
  if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return device_error(e);
  // (for the 128-wide bf16 maps the state pass compacts the softmax keys on its way: one pass over K and V)
  const bool fused_compaction = !wide && phi_k && state_compacts_softmax_keys(pl);
  if (pl.NS > 0 && !fused_compaction && (e = launch_compact(pl, k, v, ws, st)) != hipSuccess) return device_error(e);
  if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return device_error(e);
  if (pl.NL > 0 && wide) {
    if ((e = launch_wide_key_side(pl, *wide, k, v, *phi_k, ws, st)) != hipSuccess) return device_error(e);
  } else if (pl.NL > 0) {
    // (the pipelined state pass of the 128-wide bf16 maps gathers the weights from the caller's tensors itself)
    if (!state_reads_raw_weights(pl) && (e = launch_weight_prep(pl, *phi_k, false, ws, st)) != hipSuccess) return device_error(e);
    if ((e = launch_state(pl, k, v, *phi_k, ws, st)) != hipSuccess) return device_error(e);
    if (prep_q && prep_q_done && pl.CC == 0 && pl.LW == 0) {
      if ((e = launch_state_reduce_with_prep(pl, *prep_q, ws, st)) != hipSuccess) return device_error(e);
      *prep_q_done = true;
    } else if ((e = launch_state_reduce(pl, ws, st)) != hipSuccess) {
      return device_error(e);
    }
  }
  if (ev && (e = hipEventRecord(ev[2], st)) != hipSuccess) return device_error(e);
  return HA_OK;
}

}  // namespace ha

extern "C" {

ha_status hybrid_attn_validate(const ha_problem *p, const ha_feature_map *phi_q, const ha_feature_map *phi_k) {
  return ha::validate(p, phi_q, phi_k);
}

size_t hybrid_attn_workspace_bytes(const ha_problem *p, const ha_feature_map *phi_q, const ha_feature_map *phi_k) {
  if (ha::validate(p, phi_q, phi_k) != HA_OK) return 0;
  ha::Plan pl;
  ha::WidePlan wp;
  bool wide;
  return ha::full_plan(*p, phi_q, phi_k, pl, wp, wide);
}

static ha_status forward_impl(const ha_problem *p, const void *q, const void *k, const void *v,
                              const ha_feature_map *phi_q, const ha_feature_map *phi_k, void *out, float *row_den,
                              void *workspace, size_t workspace_bytes, void *hip_stream) {
  ha_status s = ha::validate(p, phi_q, phi_k);
  if (s != HA_OK) return s;
  if (!q || !k || !v || !out) return HA_ERR_NULL;
  if (!ha::aligned16(q) || !ha::aligned16(k) || !ha::aligned16(v) || !ha::aligned16(out)) return HA_ERR_ALIGN;
  ha::Plan pl;
  ha::WidePlan wp;
  bool wide;
  const size_t need = ha::full_plan(*p, phi_q, phi_k, pl, wp, wide);
  if (!workspace || workspace_bytes < need) return HA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return HA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipEvent_t *ev = ha::prof_events();
  const bool light = ev && ha::g_prof.dominant_only;
  bool prep_q_done = false;
  s = ha::run_key_side(pl, k, v, phi_k, workspace, st, light ? nullptr : ev, wide ? &wp : nullptr, wide ? nullptr : phi_q,
                       &prep_q_done);
  if (s != HA_OK) return s;
  hipError_t e;
  if (wide) {
    if ((e = ha::launch_wide_query_side(pl, wp, q, *phi_q, workspace, st)) != hipSuccess) return ha::device_error(e);
  } else if (pl.NL > 0 && !prep_q_done && (e = ha::launch_weight_prep(pl, *phi_q, true, workspace, st)) != hipSuccess) {
    return ha::device_error(e);
  }
  if (ev && (e = hipEventRecord(ev[3], st)) != hipSuccess) return ha::device_error(e);
  if ((e = ha::launch_query(pl, q, phi_q, out, row_den, workspace, st, wide ? &wp : nullptr)) != hipSuccess)
    return ha::device_error(e);
  if (ev) {
    if ((e = hipEventRecord(ev[4], st)) != hipSuccess) return ha::device_error(e);
    ++ha::g_prof.count;
  }
  return HA_OK;
}

ha_status hybrid_attn_forward(const ha_problem *p, const void *q, const void *k, const void *v,
                              const ha_feature_map *phi_q, const ha_feature_map *phi_k, void *out, void *workspace,
                              size_t workspace_bytes, void *hip_stream) {
  return forward_impl(p, q, k, v, phi_q, phi_k, out, nullptr, workspace, workspace_bytes, hip_stream);
}

// ------------------------------------------------------------------------------------------------
// Forward without a caller workspace and without any allocation: the scratch is a file-scope device array.
// In host code the array's name only stands for the symbol; its device address (one per GPU, each GPU holds its
// own copy) is looked up once per device and kept.
namespace ha {
constexpr size_t kStaticScratchBytes = (size_t)HA_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up at the first call on that device).
static hipError_t static_scratch(void **ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace ha

size_t hybrid_attn_static_scratch_bytes(void) { return ha::kStaticScratchBytes; }

ha_status hybrid_attn_forward_static(const ha_problem *p, const void *q, const void *k, const void *v,
                                     const ha_feature_map *phi_q, const ha_feature_map *phi_k, void *out,
                                     void *hip_stream) {
  ha_status s = ha::validate(p, phi_q, phi_k);
  if (s != HA_OK) return s;
  ha::Plan pl;
  ha::WidePlan wp;
  bool wide;
  // the size check is host arithmetic: a problem beyond the static array is refused before any HIP call
  if (ha::full_plan(*p, phi_q, phi_k, pl, wp, wide) > ha::kStaticScratchBytes) return HA_ERR_WORKSPACE;
  if (!q || !k || !v || !out) return HA_ERR_NULL;
  void *ws = nullptr;
  hipError_t e = ha::static_scratch(&ws);
  if (e != hipSuccess) return ha::device_error(e);
  return forward_impl(p, q, k, v, phi_q, phi_k, out, nullptr, ws, ha::kStaticScratchBytes, hip_stream);
}

ha_status hybrid_attn_profile_enable(int n_records) {
  const bool dominant_only = n_records < 0;
  if (dominant_only) n_records = -n_records;
  if (n_records > 4096) return HA_ERR_SHAPE;
  ha::Profile &pf = ha::g_prof;
  for (int i = 0; i < pf.n * 6; ++i) (void)hipEventDestroy(pf.ev[i]);
  delete[] pf.ev;
  pf.ev = nullptr;
  pf.n = pf.count = 0;
  if (n_records == 0) return HA_OK;
  pf.ev = new hipEvent_t[(size_t)n_records * 6];
  for (int i = 0; i < n_records * 6; ++i) {
    hipError_t e = hipEventCreate(&pf.ev[i]);
    if (e != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(pf.ev[j]);
      delete[] pf.ev;
      pf.ev = nullptr;
      return ha::device_error(e);
    }
  }
  pf.n = n_records;
  pf.dominant_only = dominant_only;
  return HA_OK;
}

int hybrid_attn_profile_count(void) { return ha::g_prof.count; }

ha_status hybrid_attn_profile_read(int index, float ms[5]) {
  ha::Profile &pf = ha::g_prof;
  if (!ms) return HA_ERR_NULL;
  if (pf.n == 0 || index < 0 || index >= pf.count || index < pf.count - pf.n) return HA_ERR_SHAPE;
  hipEvent_t *ev = pf.ev + (size_t)(index % pf.n) * 6;
  hipError_t e = hipEventSynchronize(ev[4]);
  if (e != hipSuccess) return ha::device_error(e);
  const int a[5] = {0, 1, 2, 3, 0}, b[5] = {1, 2, 3, 4, 4};
  for (int i = 0; i < 5; ++i) {
    if (pf.dominant_only && i != 3) {
      ms[i] = 0.f;
      continue;
    }
    if ((e = hipEventElapsedTime(&ms[i], ev[a[i]], ev[b[i]])) != hipSuccess) return ha::device_error(e);
  }
  return HA_OK;
}

ha_status hybrid_attn_linear_state(const ha_problem *p, const void *k, const void *v, const ha_feature_map *phi_k,
                                   float *state_S, float *state_z, void *workspace, size_t workspace_bytes,
                                   void *hip_stream) {
  ha_status s = ha::validate(p, phi_k, phi_k);
  if (s != HA_OK) return s;
  if (!k || !v || !state_S || !state_z || !phi_k) return HA_ERR_NULL;
  if (p->hybrid_rate == 1) return HA_ERR_SHAPE;   // no linear tokens, no state
  if (p->causal_chunk > 0 || p->local_window > 0) return HA_ERR_UNSUPPORTED;
  if (!ha::aligned16(k) || !ha::aligned16(v)) return HA_ERR_ALIGN;
  ha::Plan pl;
  ha::WidePlan wp;
  bool wide;
  const size_t need = ha::full_plan(*p, phi_k, phi_k, pl, wp, wide);
  if (!workspace || workspace_bytes < need) return HA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return HA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  s = ha::run_key_side(pl, k, v, phi_k, workspace, st, nullptr, wide ? &wp : nullptr);
  if (s != HA_OK) return s;
  const size_t BH = (size_t)pl.B * pl.H;
  char *ws = static_cast<char *>(workspace);
  hipError_t e = hipMemcpyAsync(state_S, ws + pl.off_S, BH * pl.F * pl.D * 4, hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return ha::device_error(e);
  e = hipMemcpyAsync(state_z, ws + pl.off_z, BH * pl.F * 4, hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return ha::device_error(e);
  return HA_OK;
}

ha_status hybrid_attn_mfma_probe(int random_operands, int iters, int launches, void *sink, size_t sink_bytes,
                                 double *flops_per_launch, void *hip_stream) {
  if (!sink || !flops_per_launch) return HA_ERR_NULL;
  if (iters < 1 || launches < 1 || iters > (1 << 24) || launches > (1 << 16)) return HA_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(sink) & 15u) return HA_ERR_ALIGN;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return ha::device_error(e);
  if (sink_bytes < (size_t)cus * 512 * sizeof(float)) return HA_ERR_WORKSPACE;
  // per wave and iteration: 16 instructions of 2 * 32 * 32 * 16 flops
  *flops_per_launch = (double)cus * 8.0 * (double)iters * 16.0 * 32768.0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int l = 0; l < launches; ++l) {
    e = ha::launch_mfma_probe(static_cast<float *>(sink), cus, iters, random_operands != 0, st);
    if (e != hipSuccess) return ha::device_error(e);
  }
  return HA_OK;
}

// Workspace of the loss: the larger of the two forwards' workspaces, then the reduction partials.
static size_t distill_layout(const ha_problem &p, const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                             ha::Plan &teacher, ha::Plan &student, size_t &off_partial) {
  ha_problem pt = p;
  pt.hybrid_rate = 1;
  ha::make_plan(pt, nullptr, nullptr, teacher);
  ha::WidePlan wp;
  bool wide;
  const size_t student_total = ha::full_plan(p, phi_q, phi_k, student, wp, wide);
  off_partial = ha::align256(teacher.total > student_total ? teacher.total : student_total);
  return off_partial + ha::align256(ha::l1_partial_bytes(student));
}

size_t hybrid_attn_value_distill_workspace_bytes(const ha_problem *p, const ha_feature_map *phi_q,
                                                 const ha_feature_map *phi_k) {
  if (ha::validate(p, phi_q, phi_k) != HA_OK) return 0;
  ha::Plan t, s;
  size_t off;
  return distill_layout(*p, phi_q, phi_k, t, s, off);
}

ha_status hybrid_attn_value_distill_loss(const ha_problem *p, const void *q, const void *k, const void *v,
                                         const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                                         int teacher_is_cached, void *y_teacher, void *y_student, double *loss,
                                         void *workspace, size_t workspace_bytes, void *hip_stream) {
  ha_status s = ha::validate(p, phi_q, phi_k);
  if (s != HA_OK) return s;
  if (p->causal_chunk > 0 || p->local_window > 0) return HA_ERR_UNSUPPORTED;      // the teacher of Eq. "vd_loss" is not causal
  if (!q || !k || !v || !y_teacher || !y_student || !loss) return HA_ERR_NULL;
  if (!ha::aligned16(y_teacher) || !ha::aligned16(y_student) || (reinterpret_cast<uintptr_t>(loss) & 7u)) return HA_ERR_ALIGN;
  if (y_teacher == y_student) return HA_ERR_SHAPE;
  ha::Plan pt, ps;
  size_t off_partial;
  const size_t need = distill_layout(*p, phi_q, phi_k, pt, ps, off_partial);
  if (!workspace || workspace_bytes < need) return HA_ERR_WORKSPACE;
  if (!teacher_is_cached) {
    ha_problem teacher = *p;
    teacher.hybrid_rate = 1;     // Eq. "softmax": every token is a softmax token
    s = hybrid_attn_forward(&teacher, q, k, v, nullptr, nullptr, y_teacher, workspace, workspace_bytes, hip_stream);
    if (s != HA_OK) return s;
  }
  s = hybrid_attn_forward(p, q, k, v, phi_q, phi_k, y_student, workspace, workspace_bytes, hip_stream);
  if (s != HA_OK) return s;
  double *partial = reinterpret_cast<double *>(static_cast<char *>(workspace) + off_partial);
  hipError_t e = ha::launch_l1_distance(ps, y_teacher, y_student, partial, loss, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return ha::device_error(e);
  return HA_OK;
}

// Workspace of the gradient: the loss's layout, then the backward pass's buffers.  Maps other than d -> d -> d take
// the pass-per-step backward, which brings image buffers of its own (`layered`).
struct GradLayout {
  ha::Plan teacher, student;
  ha::GradPlan gp;
  ha::WidePlan wp;
  ha::WideGradPlan wgp;
  size_t off_partial, total;
  bool layered;
};

static void grad_layout(const ha_problem &p, const ha_feature_map *phi_q, const ha_feature_map *phi_k, GradLayout &gl) {
  const size_t base = distill_layout(p, phi_q, phi_k, gl.teacher, gl.student, gl.off_partial);
  gl.layered = phi_q->d_hidden != p.d_head || phi_q->d_out != p.d_head || phi_q->w_mid;
  gl.total = base;
  if (gl.student.NL == 0) return;
  if (gl.layered) {
    ha::make_wide_plan(gl.student, base, gl.wp);
    ha::make_wide_grad_plan(gl.student, gl.wp, gl.wp.total, gl.wgp);
    gl.total = gl.wgp.total;
  } else {
    ha::make_grad_plan(gl.student, base, gl.gp);
    gl.total = gl.gp.total;
  }
}

static ha_status check_grad_maps(const ha_problem *p, const ha_feature_map *phi_q, const ha_feature_map *phi_k) {
  ha_status s = ha::validate(p, phi_q, phi_k);
  if (s != HA_OK) return s;
  if (!phi_q || !phi_k) return HA_ERR_NULL;      // also at rate 1: the shapes of the gradients come from the maps
  if (p->hybrid_rate == 1) {
    s = ha::check_map(phi_q, *p);
    if (s == HA_OK) s = ha::check_map(phi_k, *p);
    if (s != HA_OK) return s;
  }
  if (phi_q->d_out != phi_k->d_out || phi_q->d_hidden != phi_k->d_hidden) return HA_ERR_SHAPE;
  if ((phi_q->w_mid != nullptr) != (phi_k->w_mid != nullptr)) return HA_ERR_SHAPE;
  if (phi_q->w_mid && phi_q->d_mid != phi_k->d_mid) return HA_ERR_SHAPE;
  return HA_OK;
}

size_t hybrid_attn_value_distill_grad_workspace_bytes(const ha_problem *p, const ha_feature_map *phi_q,
                                                      const ha_feature_map *phi_k) {
  if (check_grad_maps(p, phi_q, phi_k) != HA_OK) return 0;
  GradLayout gl;
  grad_layout(*p, phi_q, phi_k, gl);
  return gl.total;
}

ha_status hybrid_attn_value_distill_grad(const ha_problem *p, const void *q, const void *k, const void *v,
                                         const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                                         int teacher_is_cached, int student_is_cached, void *y_teacher,
                                         void *y_student, float *row_den, double *loss,
                                         const ha_feature_map_grad *grad_q, const ha_feature_map_grad *grad_k,
                                         void *workspace, size_t workspace_bytes, void *hip_stream) {
  ha_status s = check_grad_maps(p, phi_q, phi_k);
  if (s != HA_OK) return s;
  if (p->causal_chunk > 0 || p->local_window > 0) return HA_ERR_UNSUPPORTED;
  if (!q || !k || !v || !y_teacher || !y_student || !row_den || !loss || !grad_q || !grad_k) return HA_ERR_NULL;
  for (const ha_feature_map_grad *gm : {grad_q, grad_k}) {
    if (!gm->w1 || !gm->b1 || !gm->w2 || !gm->b2) return HA_ERR_NULL;
    if (phi_q->w_mid && (!gm->w_mid || !gm->b_mid)) return HA_ERR_NULL;
    for (const float *t : {gm->w1, gm->b1, gm->w2, gm->b2, phi_q->w_mid ? gm->w_mid : nullptr, phi_q->w_mid ? gm->b_mid : nullptr})
      if (reinterpret_cast<uintptr_t>(t) & 3u) return HA_ERR_ALIGN;
  }
  if (!ha::aligned16(q) || !ha::aligned16(k) || !ha::aligned16(v) || !ha::aligned16(y_teacher) ||
      !ha::aligned16(y_student) || (reinterpret_cast<uintptr_t>(row_den) & 3u) || (reinterpret_cast<uintptr_t>(loss) & 7u))
    return HA_ERR_ALIGN;
  if (y_teacher == y_student) return HA_ERR_SHAPE;
  GradLayout gl;
  grad_layout(*p, phi_q, phi_k, gl);
  const ha::Plan &ps = gl.student;
  const size_t off_partial = gl.off_partial;
  if (!workspace || workspace_bytes < gl.total) return HA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return HA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (!teacher_is_cached) {
    ha_problem teacher = *p;
    teacher.hybrid_rate = 1;
    s = hybrid_attn_forward(&teacher, q, k, v, nullptr, nullptr, y_teacher, workspace, workspace_bytes, hip_stream);
    if (s != HA_OK) return s;
  }
  hipError_t e;
  if (!student_is_cached) {
    s = forward_impl(p, q, k, v, phi_q, phi_k, y_student, row_den, workspace, workspace_bytes, hip_stream);
    if (s != HA_OK) return s;
  } else if (ps.NL > 0) {
    // the backward pass needs S, z of the current phi_k in the workspace
    ha::Plan pf;
    ha::WidePlan wpf;
    bool wide;
    ha::full_plan(*p, phi_q, phi_k, pf, wpf, wide);
    s = ha::run_key_side(ps, k, v, phi_k, workspace, st, nullptr, wide ? &wpf : nullptr);
    if (s != HA_OK) return s;
  }
  double *partial = reinterpret_cast<double *>(static_cast<char *>(workspace) + off_partial);
  // bf16 outputs with a gradient to form: the pass that turns the two outputs into signs and row factors forms the
  // loss as well (same partial sums, same number); otherwise the loss has a pass of its own
  const bool loss_with_rows = !ps.f32 && ps.NL > 0;
  if (!loss_with_rows && (e = ha::launch_l1_distance(ps, y_teacher, y_student, partial, loss, st)) != hipSuccess)
    return ha::device_error(e);
  const size_t H = (size_t)p->H, D = (size_t)p->d_head, HD = (size_t)phi_q->d_hidden, F = (size_t)phi_q->d_out;
  const size_t DM = phi_q->w_mid ? (size_t)phi_q->d_mid : 0, KL = DM ? DM : HD;
  if (ps.NL == 0) {
    for (const ha_feature_map_grad *gm : {grad_q, grad_k}) {
      if ((e = ha::launch_fill_zero(gm->w1, H * HD * D, st)) != hipSuccess) return ha::device_error(e);
      if ((e = ha::launch_fill_zero(gm->w2, H * F * KL, st)) != hipSuccess) return ha::device_error(e);
      if ((e = ha::launch_fill_zero(gm->b1, H * HD, st)) != hipSuccess) return ha::device_error(e);
      if ((e = ha::launch_fill_zero(gm->b2, H * F, st)) != hipSuccess) return ha::device_error(e);
      if (DM && (e = ha::launch_fill_zero(gm->w_mid, H * DM * HD, st)) != hipSuccess) return ha::device_error(e);
      if (DM && (e = ha::launch_fill_zero(gm->b_mid, H * DM, st)) != hipSuccess) return ha::device_error(e);
    }
    return HA_OK;
  }
  if (gl.layered)
    e = ha::launch_wide_value_distill_backward(ps, gl.wp, gl.wgp, q, k, v, *phi_q, *phi_k, y_teacher, y_student, row_den,
                                               *grad_q, *grad_k, workspace, st, loss_with_rows ? partial : nullptr, loss);
  else
    e = ha::launch_value_distill_backward(ps, gl.gp, q, k, v, *phi_q, *phi_k, y_teacher, y_student, row_den, *grad_q, *grad_k,
                                          workspace, st, loss_with_rows ? partial : nullptr, loss);
  if (e != hipSuccess) return ha::device_error(e);
  return HA_OK;
}

const char *hybrid_attn_status_string(ha_status s) {
  switch (s) {
    case HA_OK: return "ok";
    case HA_ERR_NULL: return "a required pointer is NULL";
    case HA_ERR_SHAPE: return "invalid or inconsistent sizes";
    case HA_ERR_UNSUPPORTED: return "valid problem, but no kernel for it in this build";
    case HA_ERR_ALIGN: return "pointer or stride breaks the 16-byte alignment rule";
    case HA_ERR_WORKSPACE: return "workspace missing or too small";
    case HA_ERR_DEVICE: return "a HIP call failed (see hybrid_attn_last_device_error)";
    case HA_ERR_INFEASIBLE: return "no assignment of rates fits the budget";
  }
  return "unknown status";
}

int hybrid_attn_last_device_error(void) { return ha::g_last_device_error; }

int hybrid_attn_abi_version(void) { return 7; }

}  // extern "C"
