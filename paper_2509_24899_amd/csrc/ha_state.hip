// State pass of the hybrid-attention forward for the feature maps whose widths equal the head width (d -> d -> d):
// phi_k on the linear tokens T_L and the two cached sums of Sec. 3.1,
//     S = sum_{j in T_L} phi_k(k_j)^T v_j   (F x d),      z = sum_{j in T_L} phi_k(k_j)   (F),
// as per-chunk partial tiles that state_reduce_kernel adds up in a fixed order.  gfx950 only.
//
// One workgroup = 8 waves, two per SIMD, in two roles that meet at two barriers per 128-token tile:
//   * waves 0 - 3 evaluate phi_k, 32 token rows each, as a software pipeline: layer 1 runs two row blocks at a time
//     (two independent accumulator chains, their matrix instructions alternate); layer 2 runs two output tiles at a
//     time in steps of one hidden block, the fragments of the next step requested before the current step's matrix
//     instructions, and the softmax of the finished pair of tiles (online form: exponentials against the running
//     maximum, one factor per pair at the end) is spread over the steps of the next pair, so vector work sits under
//     matrix work.  The K rows of the next tile are requested in the middle of the current one.  phi leaves as
//     row-major bf16 (8-byte pieces) into LDS between the two barriers.
//   * waves 4 - 7 own one 32-row block of [S | z] each.  They fetch the V rows one tile ahead (global -> registers),
//     write them row-major into LDS between the two barriers, and contract [S | z] += phi^T [V | 1] over the tile
//     while the other four waves are already in the next tile's layers.  Both operands of that contraction come out
//     of LDS through the transposing 64-bit reads of gfx950 (ds_read_b64_tr_b16): four consecutive tokens of one
//     column per lane, two reads per 8-slot fragment, no 2-byte scatter anywhere; the fragments of the next two
//     16-token slices are requested while the matrix instructions of the current two run.  These waves also carry
//     the softmax-key compaction (below): it costs the feature-map waves nothing but issue slots.
// Barrier A of a tile: the contraction of the previous tile has read both LDS tiles; barrier B: both are refilled.
// Every wave of either role passes both barriers once per tile, and both roles count the same tiles.
#include "ha_device.h"
#include "ha_mlp128.h"
#include "ha_plan.h"

namespace ha {

// Row-major [token][column] bf16 tile in LDS with rows of 2 D bytes.  The 16-byte pieces of a row are XOR-swizzled by
// the row so that the transposing reads (4 rows x 32 bytes per 16 lanes) and the row-wise writes spread over the
// banks.  The swizzle only has to be the same function everywhere the tile is addressed.
template <int D>
struct RowTile {
  static constexpr int ROWB = 2 * D;        // bytes per row
  static constexpr int PPR = ROWB / 16;     // 16-byte pieces per row
  static __device__ __forceinline__ int sw(int row) { return D >= 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }
  // byte offset of 16-byte piece p of `row`
  static __device__ __forceinline__ int piece(int row, int p) { return row * ROWB + ((p ^ sw(row)) << 4); }
};

// ACT0: the output activation is the softmax over the channels (the default of the paper's maps), scheduled by hand;
// the other activations (exp, ReLU: no reduction over channels) take a plain epilogue of layer 2.
// Softmax-key compaction inside the state pass (COMPACT; bf16, the plain operator).  The softmax tokens T_S (Sec. 3.2)
// still have to reach the query kernel as matrix-core fragments (ks_frag / vs_frag, see compact_kernel): the 32-key
// blocks of a head are dealt to the head's workgroups, block chunk + j * (workgroups per head), and ride along with
// the tiles, two blocks per tile: requested before a tile's contraction, written out behind it.  K pieces pass
// through registers (a fragment piece is 16 contiguous bytes of a key row), V rows go into a small row-major LDS
// area of the wave's own (direct-to-LDS) and come out through transposing reads in the slot order the query
// kernel's second product needs.  Every K, V row of the sequence is then read by exactly one
// pass.  Key indices past the last softmax key repeat it (their logits are masked by the query kernel).
struct CompactArgs {
  bf16x8 *ks_frag, *vs_frag;   // [B*H][n_kblocks][512]
  int NS, n_kblocks;
};

// WEIGHTED (the value-distillation gradient runs this pass over all query tokens for dS = sum_i phi_q(q_i)^T g_i /
// den_i and dz = sum_i dden_i phi_q(q_i)): `k` holds the queries, `v` a dense bf16 [B*H][NL][D] tensor, token i's
// feature row is multiplied by rs[i] before it is rounded, and the "1" column becomes the pair of columns (hi, lo) of
// wp[i].
template <bool F32, bool ACT0, bool COMPACT, bool WEIGHTED = false>
__global__ __launch_bounds__(512, 1) void state_pipelined_kernel(const void *__restrict__ k, const void *__restrict__ v,
                                                                 const void *w1_src, const void *w2_src,
                                                                 const float *__restrict__ b1_all,
                                                                 const float *__restrict__ b2_all, float *__restrict__ part,
                                                                 int H, int NL, int R, int G, int CH, int P, int act,
                                                                 int64_t sb, int64_t sh, int64_t sn, int N, int CC, int nsub,
                                                                 CompactArgs ca, const float *__restrict__ rs_all = nullptr,
                                                                 const float *__restrict__ wp_all = nullptr) {
  constexpr int D = 128, HD = D, F = D, TOK = 128;
  static_assert(!(COMPACT && F32), "the compaction rides on direct-to-LDS loads of bf16 rows");
  static_assert(!(COMPACT && WEIGHTED), "the weighted pass has no softmax keys to compact");
  constexpr int KS = D / 16, HB = HD / 32, FB = F / 32, NCB = D / 32 + 1, NT = FB * NCB;
  static_assert(HB == 4 && FB == 4 && KS == 8, "the hand-placed schedule below is written for 128 -> 128 -> 128");
  typedef RowTile<D> RT;
  constexpr int ROWB = RT::ROWB, PPR = RT::PPR;
  __shared__ bf16x8 wlds[(HD * D + F * HD) / 8];
  __shared__ __align__(16) float blds[HD + F];
  __shared__ __align__(16) char phi_t[TOK * ROWB];
  __shared__ __align__(16) char v_t[TOK * ROWB];
  constexpr int CB = 2;                              // softmax-key blocks in flight per tile
  __shared__ __align__(16) char cstage[COMPACT ? CB * 4 * 2048 : 16];   // per block and wave: 16 key rows x 128 bytes of V
  __shared__ __align__(16) __bf16 et[WEIGHTED ? 2 : 1][WEIGHTED ? TOK : 8];   // hi and lo part of wp per token of the tile

  const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % H;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)h * sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int w = wave & 3;                            // index within the role
  // Weight fragments of this head: 64 KiB global -> LDS with direct-to-LDS loads, all in flight at once.
  // bf16 weights are gathered straight from the caller's row-major tensors (no preparation pass): a fragment piece is 16
  // contiguous bytes of a weight row.  For layer 2 that holds because the hidden units of every 32-block are kept in
  // a permuted order: row rho of a layer-1 fragment is weight row pi(rho), pi = swap of bits 2 and 3, so that the C
  // registers 8 s .. 8 s + 7 that feed layer 2 as its B operand hold the hidden units 16 s + 8 g .. + 7 in order
  // and the matching A fragment of W2 is a plain run of a W2 row.  fp32 weights come as prepared bf16 fragments
  // (weight_prep_kernel; W2 then in the order of the C registers, no permutation).
  constexpr bool RAWW = !F32;
  auto pi = [](int rho) { return perm_hidden(rho); };
  if constexpr (RAWW) {
    const __bf16 *w1r = static_cast<const __bf16 *>(w1_src) + (int64_t)h * HD * D;
    const __bf16 *w2r = static_cast<const __bf16 *>(w2_src) + (int64_t)h * F * HD;
    auto dma = [&](const __bf16 *gp, bf16x8 *chunk) {
      const unsigned l = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)chunk);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(gp) : "memory");
    };
    for (int c = wave; c < HB * KS; c += 8) {       // fragment (hb, ks) of W1: rows 32 hb + pi(r), columns 16 ks + 8 g ..
      const int hb = c / KS, ks = c % KS;
      dma(w1r + (int64_t)(32 * hb + pi(r)) * D + 16 * ks + 8 * g, &wlds[c * 64]);
    }
    for (int c = wave; c < FB * HB * 2; c += 8) {   // fragment (fb, hb, s) of W2: rows 32 fb + r, columns 32 hb + 16 s + 8 g ..
      const int s2 = c & 1, hb = (c >> 1) % HB, fb = (c >> 1) / HB;
      dma(w2r + (int64_t)(32 * fb + r) * HD + 32 * hb + 16 * s2 + 8 * g, &wlds[HD * D / 8 + c * 64]);
    }
  } else {
    dma_to_lds(static_cast<const bf16x8 *>(w1_src) + (int64_t)h * (HD * D / 8), &wlds[0], HD * D / 8 / 64, wave, 8, lane);
    dma_to_lds(static_cast<const bf16x8 *>(w2_src) + (int64_t)h * (F * HD / 8), &wlds[HD * D / 8], F * HD / 8 / 64, wave, 8, lane);
  }
  for (int i = tid; i < HD; i += 512) blds[i] = b1_all ? b1_all[(int64_t)h * HD + (RAWW ? (i & ~31) + pi(i & 31) : i)] : 0.f;
  for (int i = tid; i < F; i += 512) blds[HD + i] = b2_all ? b2_all[(int64_t)h * F + i] : 0.f;
  const LinearMap lmap(R, G);

  // this workgroup's range of linear tokens (see the chunking of the plan)
  int lt_begin = chunk * CH;
  int lt_end = min(lt_begin + CH, NL);
  if (CC > 0) {
    const int cc = chunk / nsub, lo = cc * CC, hi = min(lo + CC, N);
    lt_begin = lo - softmax_before(lo, R, G) + (chunk % nsub) * CH;
    lt_end = min(lt_begin + CH, hi - softmax_before(hi, R, G));
  }

  if (wave < 4) {
    // =============================== the feature map: phi_k of 32 token rows per wave ===============================
    const float *b1 = &blds[0], *b2 = &blds[HD];
    const lds_frag_ptr w1f = (lds_frag_ptr)&wlds[0], w2f = (lds_frag_ptr)&wlds[HD * D / 8];
    // phi writes: this lane owns token row tf and, per (fb, q), the 8-byte run of channels 32 fb + 8 q + 4 g .. + 3.
    // The phi tile is swizzled over sixteen rows: piece p of row t sits at p ^ psw(t), psw(t) = 4 (t % 4) + (t / 4) % 4,
    // so that the 32 rows one write instruction touches fall on 16 different 16-byte pieces (two rows per piece pair
    // with the 8-byte halves of g: conflict-free in two passes) while a transposing read still finds its four rows in
    // four different 64-byte groups.
    const int tf = w * 32 + r;
    auto psw = [](int t) { return 4 * (t & 3) + ((t >> 2) & 3); };
    int phi_base[FB][4];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
      for (int q = 0; q < 4; ++q) phi_base[fb][q] = tf * ROWB + 8 * g + (((4 * fb + q) ^ psw(tf)) << 4);
    auto load_k = [&](int t0, bf16x8 (&dst)[KS]) {
      const int tok = lmap.token(min(t0 + tf, NL - 1));   // rows past the end repeat the last linear token; masked later
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) dst[ks] = load8<F32>(k, base + (int64_t)tok * sn + 16 * ks + 8 * g);
    };
    bf16x8 xf[KS];
    load_k(lt_begin, xf);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(F32 ? 0 : KS) : "memory");     // the weight fragments are older than the K loads
    __syncthreads();                                   // weights and biases are in LDS

    for (int t0 = lt_begin; t0 < lt_end; t0 += TOK) {
      u32x4 h_hi[HB][2], h_lo[HB][2];                  // relu(W1 x + b1) as hi + lo bf16 pairs, chained order
      f32x16 u[FB];
      // the K rows of the next tile travel during layer 2 and everything behind it
      mlp128_pipelined<ACT0>(xf, w1f, w2f, b1, b2, lane, g, act, h_hi, h_lo, u, [&]() { load_k(t0 + TOK, xf); });
      if (P == 2) {
        // the paper's default degree: the upper half of the channels is squared
#pragma unroll
        for (int fb = FB / 2; fb < FB; ++fb)
#pragma unroll
          for (int x = 0; x < 16; ++x) u[fb][x] *= u[fb][x];
      } else if (P > 1) {
        // slice p = channel / Dp (0-based) gets p extra multiplications by the activation value; Dp is a multiple
        // of 8, so the power depends only on the group of four registers
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int extra = ((32 * fb + 8 * q) * P) / F;
            if (extra > 0) {
              const float t0_ = u[fb][4 * q], t1_ = u[fb][4 * q + 1], t2_ = u[fb][4 * q + 2], t3_ = u[fb][4 * q + 3];
              for (int i = 0; i < extra; ++i) {
                u[fb][4 * q] *= t0_;
                u[fb][4 * q + 1] *= t1_;
                u[fb][4 * q + 2] *= t2_;
                u[fb][4 * q + 3] *= t3_;
              }
            }
          }
      }
      float wp_tok = 0.f;
      if constexpr (WEIGHTED) {
        const int64_t ti = (int64_t)bh * NL + lmap.token(min(t0 + tf, NL - 1));
        const float rs = rs_all[ti];
        wp_tok = wp_all[ti];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
          for (int x = 0; x < 16; ++x) u[fb][x] *= rs;
      }
      if (t0 + TOK > lt_end) {                        // ragged end of the range: padded tokens add nothing
        const float keep = t0 + tf < lt_end ? 1.f : 0.f;
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
          for (int x = 0; x < 16; ++x) u[fb][x] *= keep;
      }
      // ---------------- phi -> LDS, row-major: registers 4 q .. 4 q + 3 of tile fb are channels 32 fb + 8 q + 4 g .. + 3
      typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
      u32x2 four[FB][4];
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          four[fb][q] = u32x2{pack_bf16(u[fb][4 * q], u[fb][4 * q + 1]), pack_bf16(u[fb][4 * q + 2], u[fb][4 * q + 3])};
      __syncthreads();                                 // A: the contraction of the previous tile has read phi_t
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x2 *>(phi_t + phi_base[fb][q]) = four[fb][q];
      if constexpr (WEIGHTED) {
        if (g == 0) {
          const __bf16 whi = static_cast<__bf16>(wp_tok);
          et[0][tf] = whi;
          et[1][tf] = static_cast<__bf16>(wp_tok - static_cast<float>(whi));
        }
      }
      __syncthreads();                                 // B: phi_t and v_t hold this tile
    }
    return;
  }

  // ================= the contraction over the tokens, V, and the softmax-key compaction (waves 4 .. 7) =================
  f32x16 acc[NCB];                                   // wave w owns row block w of [S | z]
#pragma unroll
  for (int i = 0; i < NCB; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[i][x] = 0.f;
  // transposing reads: lane = (group m, i, a); see ds_read_tr.  Rows T0 + i with T0 a multiple of 4, so the swizzle
  // of the row is a per-lane constant; per column block one base offset, k-steps and half-fragments are immediates
  const int tm = lane >> 4, ti = (lane >> 2) & 3, ta = lane & 3, tg = tm >> 1;
  auto tr_off = [&](int blk) {
    return (8 * tg + ti) * ROWB + (((4 * blk + 2 * (tm & 1) + (ta >> 1)) ^ RT::sw(ti)) << 4) + 8 * (ta & 1);
  };
  int tr_base[D / 32];                               // V columns 32 cb ..
#pragma unroll
  for (int blk = 0; blk < D / 32; ++blk) tr_base[blk] = tr_off(blk);
  // this wave's channel rows 32 w .. of the phi tile: rows T0 + i with T0 = 16 ks + 8 g + 4 jj, so (T0 / 4) % 4 =
  // (2 g + jj) % 4 and the two half-fragments have bases of their own
  int a_base[2];
#pragma unroll
  for (int jj = 0; jj < 2; ++jj)
    a_base[jj] = (8 * tg + ti) * ROWB + (((4 * w + 2 * (tm & 1) + (ta >> 1)) ^ (4 * ti + ((2 * tg + jj) & 3))) << 4) + 8 * (ta & 1);
  // V rows travel global -> registers one tile ahead and are written into v_t (row-major, 1 KiB = 4 rows per
  // instruction, lane -> (row, physical piece) -> logical piece of that row) between the two barriers of a tile.
  // This lane's rows are 4 RPI apart: one exact division gives the first one's group, the others follow by adding
  // the quotient and remainder of the row distance (a tile that reaches past the last linear token clamps every row
  // on its own instead).
  constexpr int RPI = 1024 / ROWB, NVI = TOK / RPI;
  const int v_row = lane / PPR, v_pp = lane % PPR;
  const int step_q = (4 * RPI) / lmap.d, step_r = (4 * RPI) % lmap.d;
  bf16x8 vreg[NVI / 4];
  auto load_v = [&](int t0) {
    const bool whole = t0 + TOK <= NL;                 // wave-uniform
    const int i0 = t0 + w * RPI + v_row;
    int grp = 0, rem = 0;
    if (whole && lmap.g != 0) {
      grp = lmap.token(i0) - i0;                       // (i0 / d + 1) g
      rem = i0 - (grp / lmap.g - 1) * lmap.d;
    }
#pragma unroll
    for (int c = 0; c < NVI / 4; ++c) {
      const int row = (4 * c + w) * RPI + v_row;
      int tok;
      if (whole) {
        tok = t0 + row + grp;
        rem += step_r;
        const bool carry = rem >= lmap.d;
        rem -= carry ? lmap.d : 0;
        grp += (step_q + (carry ? 1 : 0)) * lmap.g;
      } else {
        tok = lmap.token(min(t0 + row, NL - 1));
      }
      if constexpr (WEIGHTED) vreg[c] = static_cast<const bf16x8 *>(v)[((int64_t)bh * NL + tok) * (D / 8) + (v_pp ^ RT::sw(row))];
      else vreg[c] = load8<F32>(v, base + (int64_t)tok * sn + (v_pp ^ RT::sw(row)) * 8);
    }
  };
  auto write_v = [&]() {
#pragma unroll
    for (int c = 0; c < NVI / 4; ++c)
      *reinterpret_cast<bf16x8 *>(v_t + ((4 * c + w) * RPI + v_row) * ROWB + (v_pp << 4)) = vreg[c];
  };

  // ---- softmax-key compaction riding along (see CompactArgs)
  const int n_wg = gridDim.x;
  const int nb = COMPACT && chunk < ca.n_kblocks ? (ca.n_kblocks - chunk + n_wg - 1) / n_wg : 0;   // blocks of this workgroup
  bf16x8 kreg[CB][2];
  auto key_token = [&](int key) {                    // softmax key -> token (the first G of every R G tokens)
    key = min(key, ca.NS - 1);
    return G == 1 ? key * R : (key / G) * R * G + key % G;
  };
  typedef RowTile<64> CT;                            // the staged V slice has rows of 128 bytes
  auto compact_request = [&](int j, int c) {
    const int kb = chunk + j * n_wg;
    const int tok_k = key_token(32 * kb + r);
#pragma unroll
    for (int i = 0; i < 2; ++i)                      // K fragment chunks ks = w, w + 4: key row r, columns 16 ks + 8 g ..
      kreg[c][i] = load8<false>(k, base + (int64_t)tok_k * sn + 16 * (w + 4 * i) + 8 * g);
    // V: this wave stages keys 16 (w % 2) .. + 15 of the block, columns 64 (w / 2) .. + 63
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = 8 * i + (lane >> 3), p = (lane & 7) ^ CT::sw(row);
      const int tok_v = key_token(32 * kb + 16 * (w & 1) + row);
      const unsigned l = __builtin_amdgcn_readfirstlane(
          (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)(cstage + (c * 4 + w) * 2048 + i * 1024));
      const __bf16 *gp = static_cast<const __bf16 *>(v) + base + (int64_t)tok_v * sn + 64 * (w >> 1) + 8 * p;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(gp) : "memory");
    }
  };
  // what compact_request(j, c) fetched has landed (the caller has waited for this wave's loads): write the fragments
  auto compact_store = [&](int j, int c) {
    const int kb = chunk + j * n_wg;
    bf16x8 *kdst = ca.ks_frag + ((int64_t)bh * ca.n_kblocks + kb) * 512;
    bf16x8 *vdst = ca.vs_frag + ((int64_t)bh * ca.n_kblocks + kb) * 512;
#pragma unroll
    for (int i = 0; i < 2; ++i) kdst[(w + 4 * i) * 64 + lane] = kreg[c][i];
    // V^T fragment (rb, s) in the chained slot order: slots 4 jj .. 4 jj + 3 of lane (g, r) are keys 16 s + 8 jj + 4 g + i
    // of column 32 rb + r; rows 8 jj + 4 g + i of this wave's slice, column block rb % 2 of its 64 columns
    const char *st = cstage + (c * 4 + w) * 2048;
#pragma unroll
    for (int rbl = 0; rbl < 2; ++rbl) {
      s16x4 half[2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int row = 8 * jj + 4 * tg + ti;
        half[jj] = ds_read_tr(st, row * 128 + (((4 * rbl + 2 * (tm & 1) + (ta >> 1)) ^ CT::sw(row)) << 4) + 8 * (ta & 1));
      }
      vdst[((2 * (w >> 1) + rbl) * 2 + (w & 1)) * 64 + lane] = join(half[0], half[1]);
    }
  };

  if (lt_begin < lt_end) load_v(lt_begin);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(F32 ? 0 : NVI / 4) : "memory");   // the weight fragments are older than the V loads
  __syncthreads();                                   // weights and biases are in LDS
  int cj = 0;                                        // first of the (up to CB) blocks in flight
  for (int t0 = lt_begin; t0 < lt_end; t0 += TOK) {
    __syncthreads();                                 // A: every wave has finished the previous tile's contraction
    write_v();
    __syncthreads();                                 // B: phi_t and v_t hold this tile
    if (t0 + TOK < lt_end) load_v(t0 + TOK);
    if constexpr (COMPACT) {
#pragma unroll
      for (int c = 0; c < CB; ++c)
        if (cj + c < nb) compact_request(cj + c, c);
    }
    // ---------------- [S | z] += phi^T [V | 1] over the 128 tokens: two 16-token slices (10 matrix instructions)
    // per batch, the 20 transposing reads of the next batch placed two behind each matrix instruction
    {
      const __bf16 one = static_cast<__bf16>(r == 0 ? 1.0f : 0.0f);     // the "1" column that yields z
      const bf16x8 ones = bf16x8{one, one, one, one, one, one, one, one};
      constexpr int KB = 2, NBATCH = TOK / 16 / KB;
      constexpr int NOP = KB * (1 + D / 32);           // operand fragments per batch
      bf16x8 fr[2][NOP];                             // [buffer][(kk, operand)]: operand 0 = phi^T, 1 + cb = V
      auto rd = [&](int batch, int buf, int i) {     // both halves of one fragment: two transposing reads
        const int kk = i / (1 + D / 32), op = i % (1 + D / 32);
        const int off = (batch * KB + kk) * 16 * ROWB;
        fr[buf][i] = op == 0 ? join(ds_read_tr(phi_t, a_base[0] + off), ds_read_tr(phi_t, a_base[1] + off + 4 * ROWB))
                             : join(ds_read_tr(v_t, tr_base[op - 1] + off), ds_read_tr(v_t, tr_base[op - 1] + off + 4 * ROWB));
      };
      auto opnd = [&](int buf, int kk, int op) { return fr[buf][kk * (1 + D / 32) + op]; };
#pragma unroll
      for (int i = 0; i < NOP; ++i) rd(0, 0, i);
      HA_FENCE();
#pragma unroll
      for (int batch = 0; batch < NBATCH; ++batch) {
        const int buf = batch & 1;
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) {
          const bf16x8 a8 = opnd(buf, kk, 0);
          bf16x8 last = ones;
          if constexpr (WEIGHTED) {
            // slot i of this lane is token 16 ks + 8 g + i of the tile: eight consecutive weights, hi part for column 0,
            // lo part for column 1, nothing for the other columns
            const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
            const bf16x8 e8 = *reinterpret_cast<const bf16x8 *>(&et[r & 1][(2 * (batch * KB + kk) + g) << 3]);
            last = r < 2 ? e8 : zero;
          }
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb) {
            acc[cb] = mfma32(a8, cb < D / 32 ? opnd(buf, kk, 1 + cb) : last, acc[cb]);
            if (batch + 1 < NBATCH) rd(batch + 1, buf ^ 1, kk * NCB + cb);
            HA_FENCE();
          }
        }
      }
    }
    if constexpr (COMPACT) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the staged V rows of the blocks have landed
#pragma unroll
      for (int c = 0; c < CB; ++c)
        if (cj + c < nb) compact_store(cj + c, c);
      cj += CB;
    }
  }
  if constexpr (COMPACT) {
    // blocks the tiles did not cover (few linear tokens per softmax key, or a short last chunk): two at a time
    for (; cj < nb; cj += CB) {
#pragma unroll
      for (int c = 0; c < CB; ++c)
        if (cj + c < nb) compact_request(cj + c, c);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int c = 0; c < CB; ++c)
        if (cj + c < nb) compact_store(cj + c, c);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the staging area is requested again right away
    }
  }
  {
    float *dst = part + ((int64_t)bh * gridDim.x + chunk) * NT * 1024 + (int64_t)w * NCB * 1024;
#pragma unroll
    for (int i = 0; i < NCB; ++i)
#pragma unroll
      for (int x = 0; x < 16; ++x) dst[i * 1024 + x * 64 + lane] = acc[i][x];
  }
}

hipError_t launch_state_pipelined(const Plan &pl, const void *k, const void *v, const ha_feature_map &fm, void *ws,
                                  hipStream_t st) {
  dim3 grid(pl.n_chunks, pl.B * pl.H);
  char *wsb = static_cast<char *>(ws);
  // bf16 weights are read in place; fp32 ones as the bf16 fragments weight_prep_kernel left in the workspace
  const void *w1f = pl.f32 ? static_cast<const void *>(wsb + pl.off_w1k) : fm.w1;
  const void *w2f = pl.f32 ? static_cast<const void *>(wsb + pl.off_w2k) : fm.w2;
  float *part = reinterpret_cast<float *>(wsb + pl.off_part);
  CompactArgs ca;
  ca.ks_frag = reinterpret_cast<bf16x8 *>(wsb + pl.off_ks);
  ca.vs_frag = reinterpret_cast<bf16x8 *>(wsb + pl.off_vs);
  ca.NS = pl.NS;
  ca.n_kblocks = pl.n_kblocks;
  const bool cmp = state_compacts_softmax_keys(pl);
#define HA_STATE(F32, ACT0, CMP) \
  state_pipelined_kernel<F32, ACT0, CMP><<<grid, 512, 0, st>>>(k, v, w1f, w2f, fm.b1, fm.b2, part, pl.H, pl.NL, pl.R, pl.G, pl.CH, \
                                                              pl.P, pl.act_k, pl.sb, pl.sh, pl.sn, pl.N, pl.CC, pl.nsub, ca)
  if (pl.act_k == HA_ACT_SOFTMAX) {
    if (pl.f32) HA_STATE(true, true, false);
    else if (cmp) HA_STATE(false, true, true);
    else HA_STATE(false, true, false);
  } else {
    if (pl.f32) HA_STATE(true, false, false);
    else if (cmp) HA_STATE(false, false, true);
    else HA_STATE(false, false, false);
  }
#undef HA_STATE
  return hipGetLastError();
}

// The weighted pass over all query tokens (see WEIGHTED): partial tiles into `part`, chunks of CH tokens.
hipError_t launch_state_pipelined_weighted(const Plan &pl, const void *q, const void *gsign, const float *rs, const float *wp,
                                           const ha_feature_map &fm, const void *w1f, const void *w2f, float *part, int CH,
                                           int n_chunks, hipStream_t st) {
  dim3 grid(n_chunks, pl.B * pl.H);
  // bf16 weights are read in place; fp32 ones as the prepared bf16 fragments the caller hands in
  const void *w1 = pl.f32 ? w1f : fm.w1;
  const void *w2 = pl.f32 ? w2f : fm.w2;
  CompactArgs ca = {nullptr, nullptr, 0, 0};
#define HA_WSTATE(F32, ACT0) \
  state_pipelined_kernel<F32, ACT0, false, true><<<grid, 512, 0, st>>>(q, gsign, w1, w2, fm.b1, fm.b2, part, pl.H, pl.N, 0, 1, CH, pl.P, \
                                                                      pl.act_q, pl.sb, pl.sh, pl.sn, pl.N, 0, 1, ca, rs, wp)
  if (pl.act_q == HA_ACT_SOFTMAX) { if (pl.f32) HA_WSTATE(true, true); else HA_WSTATE(false, true); }
  else { if (pl.f32) HA_WSTATE(true, false); else HA_WSTATE(false, false); }
#undef HA_WSTATE
  return hipGetLastError();
}

}  // namespace ha
