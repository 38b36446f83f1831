// Host-side plan of one forward: tile shapes, grid sizes and the layout of the caller's workspace.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/hybrid_attn.h"

namespace ha {

struct Plan {
  // problem
  int B, H, N, D, HD, F, R, NS, NL, P, act_q, act_k;
  int G;                 // granularity of the token split (1: per token, Sec. 3.2)
  int CC, n_cc, nsub;    // chunk-causal variant: chunk length in tokens (0: off), number of chunks, state-pass
                         // workgroups per chunk.  Local-window variant: CC = the query tile, one state per tile
  int LW;                // local-window variant: window in tokens on either side of the query's tile (0: off)
  int DM;   // width of the second hidden layer of a three-layer feature map, 0 for two layers
  bool f32;
  int64_t sb, sh, sn;
  float scale;
  // softmax part: KT = block_size (the key fragments are padded to whole multiples of it), QT queries per
  // workgroup of the query kernel (2 x block_size: block_size / 16 waves of 32 queries), 32-key blocks
  int KT, QT, n_qtiles, n_ktiles, n_kblocks;
  // state pass: CH linear tokens per workgroup, partial tiles per chunk
  int CH, n_chunks, n_state_tiles;
  // workspace byte offsets (all multiples of 256)
  size_t off_w1q, off_w2q, off_w1k, off_w2k, off_ks, off_vs, off_part, off_S, off_z, off_sthi, off_stlo, total;
};

// Workspace of the value-distillation gradient beyond the forward's: operand fragments of W2^T, S and dS, the
// per-row factors, the sign tensor and the partial tiles of the two gradient passes.
struct GradPlan {
  int CHq, n_chunks_q, CHk, n_chunks_k, tiles_per_set;
  size_t off_w2tq, off_w2tk, off_shi, off_slo, off_dS, off_dz, off_dshi, off_dslo, off_gsign, off_rs, off_wp, off_part, total;
};

// Workspace of the layer-by-layer path for feature maps beyond the fused kernels' widths (beyond the forward's):
// hidden activations (hi + lo), fp32 pre-activations, phi, and for the queries n = phi_q S and e = phi_q . z.
struct WidePlan {
  int n_tb_q, n_tb_k;      // 32-token blocks of the query tokens / the linear key tokens
  size_t off_w1, off_wm, off_w2;   // weight fragments of the map being evaluated (key side, then query side)
  size_t off_hhi, off_hlo, off_h2hi, off_h2lo, off_u, off_stat, off_phi, off_lin, off_e, total;
};

// Number of softmax tokens among the first t tokens: the first G of every R G tokens (Sec. 3.2 with G = 1).
static __host__ __device__ inline int softmax_before(int t, int R, int G) {
  if (R == 0) return 0;
  const int grp = R * G, rem = t % grp;
  return (t / grp) * G + (rem < G ? rem : G);
}

// Workspace of the value-distillation gradient of maps that take the layer-by-layer path (beyond WidePlan's).
struct WideGradPlan {
  int CHq, n_chunks_q, CHk, n_chunks_k;
  size_t off_wt, off_wtm, off_dpre2, off_shi, off_slo, off_dS, off_dz, off_dshi, off_dslo, off_gsign, off_rs, off_wp, off_tdt, off_pdot, off_du,
      off_dpre, off_part, total;
};

// Which kernels read bf16 feature-map weights straight from the caller's tensors (no weight_prep_kernel launch needed).
static inline bool state_uses_pipelined_kernel(const Plan &pl) { return pl.D == 128 && pl.HD == 128 && pl.F == 128; }
static inline bool state_reads_raw_weights(const Plan &pl) { return state_uses_pipelined_kernel(pl) && !pl.f32; }
// ... and compacts the softmax keys on the way (no compact_kernel launch): bf16, the plain operator with both kinds of tokens
static inline bool state_compacts_softmax_keys(const Plan &pl) {
  return state_uses_pipelined_kernel(pl) && !pl.f32 && pl.CC == 0 && pl.LW == 0 && pl.NS > 0 && pl.NL > 0 && pl.n_chunks > 0;
}

// Fills `pl` from a validated problem.  Pure host arithmetic.
void make_plan(const ha_problem &p, const ha_feature_map *phi_q, const ha_feature_map *phi_k, Plan &pl);

// Kernel launchers (ha_kernels.hip).  Each enqueues on `st` and returns the launch status.
hipError_t launch_weight_prep(const Plan &pl, const ha_feature_map &fm, bool is_query, void *ws, hipStream_t st);
hipError_t launch_compact(const Plan &pl, const void *k, const void *v, void *ws, hipStream_t st);
hipError_t launch_state(const Plan &pl, const void *k, const void *v, const ha_feature_map &phi_k, void *ws,
                        hipStream_t st);
hipError_t launch_state_pipelined(const Plan &pl, const void *k, const void *v, const ha_feature_map &phi_k, void *ws,
                                  hipStream_t st);
hipError_t launch_state_pipelined_weighted(const Plan &pl, const void *q, const void *gsign, const float *rs, const float *wp,
                                           const ha_feature_map &fm, const void *w1f, const void *w2f, float *part, int CH,
                                           int n_chunks, hipStream_t st);   // ha_state.hip: the d -> d -> d maps
hipError_t launch_weighted_state(const Plan &pl, const void *q, const void *gsign, const float *rs, const float *wp,
                                 const ha_feature_map &fm, const void *w1f, const void *w2f, float *part, int CH,
                                 int n_chunks, hipStream_t st);
hipError_t launch_state_reduce(const Plan &pl, void *ws, hipStream_t st);
// the plain reduction (no prefix / window states) together with the re-ordering of phi_q's weights, one launch
hipError_t launch_state_reduce_with_prep(const Plan &pl, const ha_feature_map &phi_q, void *ws, hipStream_t st);
hipError_t launch_query(const Plan &pl, const void *q, const ha_feature_map *phi_q, void *out, float *row_den, void *ws,
                        hipStream_t st, const WidePlan *wide = nullptr);
// ha_wide.hip
void make_wide_plan(const Plan &pl, size_t base_off, WidePlan &wp);
hipError_t launch_wide_key_side(const Plan &pl, const WidePlan &wp, const void *k, const void *v, const ha_feature_map &phi_k,
                                void *ws, hipStream_t st);
hipError_t launch_wide_query_side(const Plan &pl, const WidePlan &wp, const void *q, const ha_feature_map &phi_q, void *ws,
                                  hipStream_t st);
size_t l1_partial_bytes(const Plan &pl);
hipError_t launch_l1_distance(const Plan &pl, const void *ya, const void *yb, double *partial, double *loss,
                              hipStream_t st);
constexpr int kL1Parts = 64;   // partial sums of the loss per (batch, head)
hipError_t launch_l1_final(const Plan &pl, const double *partial, double *loss, hipStream_t st);
// ha_grad.hip
void make_grad_plan(const Plan &pl, size_t base_off, GradPlan &gp);
hipError_t launch_fill_zero(float *p, size_t n, hipStream_t st);
hipError_t launch_value_distill_backward(const Plan &pl, const GradPlan &gp, const void *q, const void *k, const void *v,
                                         const ha_feature_map &phi_q, const ha_feature_map &phi_k, const void *y_teacher,
                                         const void *y_student, const float *row_den, const ha_feature_map_grad &gq,
                                         const ha_feature_map_grad &gk, void *ws, hipStream_t st, double *l1_partial = nullptr,
                                         double *loss = nullptr);
// l1_partial / loss given (bf16 io only): the pass over the two outputs also forms the loss (the partial sums of
// l1_partial_kernel, bit for bit), and the final sum is launched behind it
hipError_t launch_vd_rows(const Plan &pl, const void *y_teacher, const void *y_student, const float *row_den, void *gsign,
                          float *rs, float *wp, hipStream_t st, double *l1_partial = nullptr, double *loss = nullptr);
hipError_t launch_natural_frags(const float *M, void *hi, void *lo, int rows, int cols, int n_mat, hipStream_t st);
// ha_wide.hip / ha_wide_grad.hip
hipError_t launch_wide_map(const Plan &pl, const WidePlan &wp, const void *x, const ha_feature_map &fm, bool is_query, void *ws,
                           hipStream_t st);
void make_wide_grad_plan(const Plan &pl, const WidePlan &wp, size_t base_off, WideGradPlan &gp);
hipError_t launch_wide_value_distill_backward(const Plan &pl, const WidePlan &wp, const WideGradPlan &gp, const void *q,
                                              const void *k, const void *v, const ha_feature_map &phi_q,
                                              const ha_feature_map &phi_k, const void *y_teacher, const void *y_student,
                                              const float *row_den, const ha_feature_map_grad &gq, const ha_feature_map_grad &gk,
                                              void *ws, hipStream_t st, double *l1_partial = nullptr, double *loss = nullptr);
hipError_t launch_mfma_probe(float *sink, int workgroups, int iters, int random_operands, hipStream_t st);

}  // namespace ha
