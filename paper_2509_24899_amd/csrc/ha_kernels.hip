// HIP kernels of the hybrid-attention forward (Attention Surgery, Sec. 3.2, Eq. "hybrid"), gfx950.
//
//   weight_prep_kernel   MLP weights -> bf16 A-operand fragments (once per call, tiny)
//   compact_kernel       softmax tokens T_S (every R-th token, Sec. 3.2): K_S and V_S gathered into
//                        matrix-core fragment order, zero padded to whole key tiles
//   state_kernel         linear tokens T_L: phi_k(k_j), then partial S = sum phi_k(k_j)^T v_j and
//                        z = sum phi_k(k_j) per chunk of tokens (Sec. 3.1: the two cached sums)
//   state_reduce_kernel  fixed-order sum of the partials -> S, z (fp32) and S^T as hi/lo bf16 fragments
//   (ha_query.hip)       query kernel, per 32-query column block: flash-style loop over K_S/V_S with
//                        online maximum c_i, then phi_q(q_i), phi_q(q_i).S, phi_q(q_i).z and the merge
//                        (a_i + n_i) / (l_i + e_i) of Eq. "hybrid"
//   l1_partial_kernel, l1_final_kernel   || y - y_hat ||_1 of the value-distillation loss (Sec. 3.3)
//   mfma_probe_kernel    measurement aid: matrix instructions only
//
// All products are computed transposed (keys x queries, channels x tokens) so that one lane owns one
// query / token column: row maxima and sums are in-lane plus one exchange with lane ^ 32.
#include <type_traits>

#include "ha_device.h"
#include "ha_plan.h"

namespace ha {

// ------------------------------------------------------------------------------------------------
// weight_prep_kernel: grid (ceil(max(HD*D, F*HD) / 256), H); see weight_prep_body
template <bool F32>
__global__ __launch_bounds__(256) void weight_prep_kernel(const void *__restrict__ w1, const void *__restrict__ w2,
                                                          __bf16 *__restrict__ w1f, __bf16 *__restrict__ w2f,
                                                          int D, int HD, int F) {
  weight_prep_body<F32>(w1, w2, w1f, w2f, D, HD, F, blockIdx.y, blockIdx.x * 256 + threadIdx.x);
}

// ------------------------------------------------------------------------------------------------
// compact_kernel: grid (n_kblocks, B*H); one workgroup builds one 32-key block of both fragment arrays.
//   ks_frag[bh][kb][ks][lane]          = K[token(32kb + r)][16ks + 8g .. +7]
//   vs_frag[bh][kb][rb][s][lane][t]    = V[token(32kb + crow(8s + t, g))][32rb + r]
// token(key) = key * R, or with groups of G tokens (key / G) R G + key % G; keys >= NS are zero padding.
template <int D, bool F32>
__global__ __launch_bounds__(256) void compact_kernel(const void *__restrict__ k, const void *__restrict__ v,
                                                      bf16x8 *__restrict__ ks_frag, bf16x8 *__restrict__ vs_frag,
                                                      int H, int NS, int R, int G, int n_kblocks, int64_t sb,
                                                      int64_t sh, int64_t sn) {
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int FRAG = D * 4;           // bf16x8 per 32-key block (= D*32*2/16)
  __shared__ __align__(16) __bf16 vt[32][D + 8];
  const int kb = blockIdx.x, bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)(bh % H) * sh;
  bf16x8 *kdst = ks_frag + ((int64_t)bh * n_kblocks + kb) * FRAG;
  bf16x8 *vdst = vs_frag + ((int64_t)bh * n_kblocks + kb) * FRAG;
  for (int c = threadIdx.x; c < 32 * CPR; c += 256) {
    const int r = c / CPR, c8 = c % CPR;
    const int key = kb * 32 + r;
    bf16x8 kv = {0, 0, 0, 0, 0, 0, 0, 0}, vv = kv;
    if (key < NS) {
      const int64_t off = base + (int64_t)(G == 1 ? key * R : (key / G) * R * G + key % G) * sn + c8 * 8;
      kv = load8<F32>(k, off);
      vv = load8<F32>(v, off);
    }
    kdst[(c8 >> 1) * 64 + (c8 & 1) * 32 + r] = kv;
    *reinterpret_cast<bf16x8 *>(&vt[r][c8 * 8]) = vv;
  }
  __syncthreads();
  for (int c = threadIdx.x; c < FRAG; c += 256) {
    const int lane = c & 63, rbs = c >> 6;
    const int rb = rbs >> 1, s = rbs & 1, g = lane >> 5, r = lane & 31;
    bf16x8 o;
#pragma unroll
    for (int t = 0; t < 8; ++t) o[t] = vt[16 * s + crow(t, g)][32 * rb + r];
    vdst[c] = o;
  }
}

// ------------------------------------------------------------------------------------------------
// state_kernel: grid (n_chunks, B*H), 4 waves.  A chunk is CH linear tokens, walked in tiles of 128.
// Per tile every wave runs the phi_k MLP on its 32 tokens (tokens are C columns), the four waves
// park phi_k(k)^T and V^T in LDS with tokens contiguous, then the output tiles of
// [S | z] = phi_k(K)^T [V | 1] are dealt round-robin to the waves and contracted over the tokens.
// Partial tiles go to part[bh][chunk][tile][v][lane] (fp32).
//
// Global loads run ahead of their use: the V rows of tile t are requested before its MLP starts and
// the K rows of tile t+1 as soon as layer 1 of tile t is done with the current ones.  Both LDS arrays hold [feature row][token] with the 8-token (16 B)
// blocks of a row XOR-swizzled by ((row / 8) % 4) * 2, which spreads the 2-byte transposing writes
// and the 16-byte operand reads over all banks.
//
// WEIGHTED (the value-distillation gradient reuses this pass for dS = sum_i phi_q(q_i)^T g_i / den_i and
// dz = sum_i dden_i phi_q(q_i) over all query tokens): `k` holds the queries, `v` a dense bf16 [B*H][NL][D]
// tensor, token i's feature row is multiplied by rs[i] before it is rounded, and the "1" column becomes the pair
// of columns (hi, lo) of wp[i].
template <int D, int HD, int F, bool F32, bool WEIGHTED = false>
__global__ __launch_bounds__(256, 1) void state_kernel(const void *__restrict__ k, const void *__restrict__ v,
                                                       const bf16x8 *w1f_all, const bf16x8 *w2f_all,
                                                       const float *__restrict__ b1_all, const float *__restrict__ b2_all,
                                                       float *__restrict__ part, int H, int NL, int R, int G, int CH, int P,
                                                       int act, int64_t sb, int64_t sh, int64_t sn,
                                                       const float *__restrict__ rs_all = nullptr,
                                                       const float *__restrict__ wp_all = nullptr, int N = 0, int CC = 0,
                                                       int nsub = 1) {
  constexpr int TOK = 128, PITCH = TOK + 8;
  constexpr int KS = D / 16, FB = F / 32, NCB = D / 32 + 1, NT = FB * NCB;
  constexpr int RPW = FB >= 4 ? FB / 4 : 1;   // row blocks of [S | z] per wave
  constexpr int GW = FB / RPW;                // waves that take part in the state contraction
  constexpr int TPW = RPW * NCB;              // output tiles per such wave
  constexpr int CG = D / 32;                  // groups of four 16-byte chunks per V row
  constexpr int VPT = (TOK / 16) * CG / 4;    // V chunks per thread per tile
  // the MLP weight fragments of this head live in LDS when they fit next to the two transposing arrays
  constexpr bool WLDS = (HD * D + F * HD) * 2 <= 64 * 1024;
  // Wider maps: the weights do not fit next to the two transposing arrays, but those are idle while the MLP runs.
  // One raw area serves both: per tile W1 and the first half of W2 are staged into it (direct-to-LDS, one fetch
  // per workgroup instead of one per wave), the second half of W2 follows once layer 1 is done, and only then
  // the area becomes phi^T and V^T.
  constexpr bool WIDE = F > 128;
  constexpr int NW1 = HD * D / 8, NW2 = F * HD / 8;            // bf16x8 per head
  constexpr int RAW = WIDE ? (NW1 + NW2 / 2 > (F + D) * PITCH / 8 ? NW1 + NW2 / 2 : (F + D) * PITCH / 8) : 1;
  static_assert(!WIDE || (NW2 / 2 <= NW1 && (F / 32) % 2 == 0 && RAW * 16 <= 150 * 1024), "staging plan does not fit");
  __shared__ __align__(16) __bf16 ft_s[WIDE ? 1 : F][PITCH];
  __shared__ __align__(16) __bf16 vt_s[WIDE ? 1 : D][PITCH];
  __shared__ bf16x8 raw[RAW];
  __shared__ bf16x8 wlds[WLDS ? (HD * D + F * HD) / 8 : 1];
  __shared__ __align__(16) __bf16 et[WEIGHTED ? 2 : 1][WEIGHTED ? PITCH : 8];
  static_assert(!WEIGHTED || F <= 128, "the weighted pass is built for the narrow maps only");
  const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % H;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)h * sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, kept scalar
  const bf16x8 *w1g = w1f_all + (int64_t)h * (HD * D / 8);
  const bf16x8 *w2g = w2f_all + (int64_t)h * (F * HD / 8);
  if constexpr (WLDS) {
    for (int i = tid; i < HD * D / 8; i += 256) wlds[i] = w1g[i];
    for (int i = tid; i < F * HD / 8; i += 256) wlds[HD * D / 8 + i] = w2g[i];
    // visible to all waves after the first barrier inside the tile loop; layer 1 of the first tile
    // must not start before that, so synchronise once here
    __syncthreads();
  }
  std::conditional_t<WLDS, lds_frag_ptr, GlobalFrags> w1f, w2f;
  if constexpr (WLDS) {
    w1f = (lds_frag_ptr)&wlds[0];
    w2f = (lds_frag_ptr)&wlds[HD * D / 8];
  } else {
    w1f = global_frags(w1g, HD * D * 2);
    w2f = global_frags(w2g, F * HD * 2);
  }
  // the biases of this head sit in LDS (zeros when absent): their reads queue up with the weight reads
  // instead of exposing a vector-memory round trip in front of every chain of matrix instructions
  __shared__ float blds[HD + F];
  for (int i = tid; i < HD; i += 256) blds[i] = b1_all ? b1_all[(int64_t)h * HD + i] : 0.f;
  for (int i = tid; i < F; i += 256) blds[HD + i] = b2_all ? b2_all[(int64_t)h * F + i] : 0.f;
  __syncthreads();
  const float *b1 = &blds[0];
  const float *b2 = &blds[HD];
  const int Dp = F / P;
  const LinearMap lmap(R, G);

  // wave w < GW owns row blocks fb = w*RPW .. + RPW - 1 of [S | z] with all NCB column blocks each
  // (tile = fb * NCB + cb), so every A fragment read from LDS feeds NCB products
  f32x16 acc[TPW];
#pragma unroll
  for (int i = 0; i < TPW; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[i][x] = 0.f;

  // LDS addressing.  Element (row, token) sits at row * PITCH + (((token / 8) ^ sw(row)) * 8 + token % 8),
  // sw(row) = ((row / 8) % 4) * 2.
  //  - phi writes: this lane owns token tf = 32 w + r and rows 32 fb + 8 q + 4 g + e; sw = 2 q is known
  //    at compile time, so four column offsets (one per q) cover every write
  //  - V writes: per pass this lane owns one 16-byte chunk = rows 8 c8 .. 8 c8 + 7 of one token
  //  - operand reads: rows 32 * blk + r, 16-byte token blocks 2 ks + g
  const int tf = w * 32 + r;
  int fcol[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) fcol[q] = (4 * g) * PITCH + ((((tf >> 3) ^ (2 * q)) << 3) | (tf & 7));
  const int vsw = (lane >> 4) << 1;                       // sw of rows 8 c8 + i, c8 % 4 = lane / 16
  const int vrow0 = 8 * (lane >> 4) * PITCH;
  const int rsw = ((r >> 3) & 3) << 1;                    // sw of operand rows 32 blk + r
  __bf16 *ftp = WIDE ? reinterpret_cast<__bf16 *>(&raw[0]) : &ft_s[0][0];
  __bf16 *vtp = WIDE ? reinterpret_cast<__bf16 *>(&raw[0]) + F * PITCH : &vt_s[0][0];

  // this workgroup's range of linear tokens: chunk number `chunk` of CH tokens, or (chunk-causal variant) piece
  // chunk % nsub of the linear tokens of causal chunk chunk / nsub
  int lt_begin = chunk * CH;
  int lt_end = min(lt_begin + CH, NL);
  if (CC > 0) {
    const int cc = chunk / nsub, lo = cc * CC, hi = min(lo + CC, N);
    lt_begin = lo - softmax_before(lo, R, G) + (chunk % nsub) * CH;
    lt_end = min(lt_begin + CH, hi - softmax_before(hi, R, G));
  }
  // rows past the end of T_L are clamped to the last linear token (valid memory) and masked later
  auto load_k = [&](int t0, bf16x8 (&dst)[KS]) {
    const int tok = lmap.token(min(t0 + tf, NL - 1));
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) dst[ks] = load8<F32>(k, base + (int64_t)tok * sn + 16 * ks + 8 * g);
  };
  bf16x8 xf[KS];
  load_k(lt_begin, xf);
  for (int t0 = lt_begin; t0 < lt_end; t0 += TOK) {
    // V rows of this tile: pass p of wave w covers tokens 16 ((4p + w) % 8) .. + 15 and the four
    // 16-byte chunks 4 (p / 2) .. + 3 of each (64 contiguous bytes per row)
    // (wide maps: the MLP needs the registers, so V is requested only once the hidden activations are dead)
    bf16x8 vreg[VPT];
    auto load_v = [&]() {
#pragma unroll
      for (int p = 0; p < VPT; ++p) {
        const int trow = 16 * ((4 * p + w) & 7) + (lane & 15), c8 = 4 * (p >> 1) + (lane >> 4);
        const int tok = lmap.token(min(t0 + trow, NL - 1));
        if constexpr (WEIGHTED) vreg[p] = static_cast<const bf16x8 *>(v)[((int64_t)bh * NL + tok) * (D / 8) + c8];
        else vreg[p] = load8<F32>(v, base + (int64_t)tok * sn + c8 * 8);
      }
    };
    if constexpr (!WIDE) load_v();
    __builtin_amdgcn_sched_barrier(0);
    // phi_k on this wave's 32 tokens; the K rows of the next tile are requested as soon as layer 1
    // has consumed the current ones
    {
      bf16x8 phi[FB][2];
      {
        bf16x8 h_hi[HD / 32][2], h_lo[HD / 32][2];
        if constexpr (WIDE) {
          // the previous tile's contraction is over (barrier at the end of the loop body): the area is free
          dma_to_lds(w1g, &raw[0], NW1 / 64, w, 4, lane);
          dma_to_lds(w2g, &raw[NW1], NW2 / 2 / 64, w, 4, lane);
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();
          feature_mlp_layer1<D, HD, true>(xf, (lds_frag_ptr)&raw[0], b1, lane, g, h_hi, h_lo);
        } else {
          feature_mlp_layer1<D, HD, true>(xf, w1f, b1, lane, g, h_hi, h_lo);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_k(t0 + TOK, xf);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (WIDE) {
          PhiState<FB> st;
          feature_layer2_phi_tiles<HD, F, 0, FB / 2, false>(h_hi, h_lo, (lds_frag_ptr)&raw[NW1], 0, b2, lane, g, act, P, Dp, st,
                                                           phi);
          __syncthreads();                                  // every wave is done with W1: the second half of W2 replaces it
          dma_to_lds(w2g + NW2 / 2, &raw[0], NW2 / 2 / 64, w, 4, lane);
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();
          feature_layer2_phi_tiles<HD, F, FB / 2, FB, false>(h_hi, h_lo, (lds_frag_ptr)&raw[0], (FB / 2) * (HD / 32) * 2, b2,
                                                            lane, g, act, P, Dp, st, phi);
          feature_phi_finish<F>(st, act, P, Dp, phi);
        } else {
          f32x16 u[FB];
          feature_mlp_layer2<HD, F, true>(h_hi, h_lo, w2f, b2, lane, g, u);
          feature_activation<FB>(u, g, act, P, Dp);
          float rs = 1.f;
          if constexpr (WEIGHTED) rs = rs_all[(int64_t)bh * NL + lmap.token(min(t0 + tf, NL - 1))];
#pragma unroll
          for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {
              f32x8 t8;
#pragma unroll
              for (int i = 0; i < 8; ++i) t8[i] = WEIGHTED ? u[fb][8 * sp + i] * rs : u[fb][8 * sp + i];
              phi[fb][sp] = __builtin_convertvector(t8, bf16x8);
            }
        }
      }
      if constexpr (WIDE) {
        load_v();
        __syncthreads();                                    // the weights have been read by every wave: the area becomes phi^T | V^T
      }
      if (t0 + TOK > lt_end) {                             // ragged end of the range: padded tokens add nothing
        const bool valid = t0 + tf < lt_end;
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
          for (int sp = 0; sp < 2; ++sp) phi[fb][sp] = valid ? phi[fb][sp] : zero;
      }
      // element (sp, i) of a tile is register x = 8 sp + i, i.e. row 32 fb + crow(x, g)
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int x = 0; x < 16; ++x)
          ftp[(32 * fb + 8 * (x >> 2) + (x & 3)) * PITCH + fcol[x >> 2]] = phi[fb][x >> 3][x & 7];
    }
#pragma unroll
    for (int p = 0; p < VPT; ++p) {
      const int trow = 16 * ((4 * p + w) & 7) + (lane & 15);
      const int col = (((trow >> 3) ^ vsw) << 3) | (trow & 7);
#pragma unroll
      for (int i = 0; i < 8; ++i) vtp[(32 * (p >> 1) + i) * PITCH + vrow0 + col] = vreg[p][i];
    }
    if constexpr (WEIGHTED) {
      if (g == 0) {
        const float wp = wp_all[(int64_t)bh * NL + lmap.token(min(t0 + tf, NL - 1))];
        const __bf16 whi = static_cast<__bf16>(wp);
        et[0][tf] = whi;
        et[1][tf] = static_cast<__bf16>(wp - static_cast<float>(whi));
      }
    }
    __syncthreads();
    if (w < GW) {
      const __bf16 one = static_cast<__bf16>(r == 0 ? 1.0f : 0.0f);     // the "1" column that yields z
      const bf16x8 ones = bf16x8{one, one, one, one, one, one, one, one};
      // two 16-token slices at a time: all their fragments are requested before the matrix instructions that
      // use them (one wave per SIMD: nothing else hides the LDS latency)
      constexpr int KB = 2;
#pragma unroll
      for (int ks0 = 0; ks0 < TOK / 16; ks0 += KB) {
        bf16x8 af[KB][RPW], bfr[KB][D / 32], ew[KB];
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) {
          const int col = ((2 * (ks0 + kk) + g) ^ rsw) << 3;
          if constexpr (WEIGHTED) {
            const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
            const bf16x8 e8 = *reinterpret_cast<const bf16x8 *>(&et[r & 1][(2 * (ks0 + kk) + g) << 3]);
            ew[kk] = r < 2 ? e8 : zero;
          } else {
            ew[kk] = ones;
          }
#pragma unroll
          for (int rp = 0; rp < RPW; ++rp)
            af[kk][rp] = *reinterpret_cast<const bf16x8 *>(&ftp[(32 * (w * RPW + rp) + r) * PITCH + col]);
#pragma unroll
          for (int cb = 0; cb < D / 32; ++cb)
            bfr[kk][cb] = *reinterpret_cast<const bf16x8 *>(&vtp[(32 * cb + r) * PITCH + col]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KB; ++kk)
#pragma unroll
          for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
              acc[rp * NCB + cb] = mfma32(af[kk][rp], cb < D / 32 ? bfr[kk][cb] : ew[kk], acc[rp * NCB + cb]);
      }
    }
    __syncthreads();
  }
  if (w < GW) {
    float *dst = part + ((int64_t)bh * gridDim.x + chunk) * NT * 1024 + (int64_t)w * TPW * 1024;
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
      for (int x = 0; x < 16; ++x) dst[i * 1024 + x * 64 + lane] = acc[i][x];
  }
}

// ------------------------------------------------------------------------------------------------
// state_reduce_kernel: grid (NT*1024/256, B*H).  Sums the chunk partials in chunk order (bitwise
// reproducible), writes S [F][D] and z [F] in fp32, and S^T split into hi + lo bf16 in the
// A-operand order of the query kernel:  st[bh][rb][fb][s][lane][t] = S[32fb + crow(8s + t, g)][32rb + r].
static __device__ __forceinline__ void state_reduce_body(const float *__restrict__ part, float *__restrict__ S,
                                                         float *__restrict__ z, __bf16 *__restrict__ st_hi,
                                                         __bf16 *__restrict__ st_lo, int D, int F, int n_chunks, int bh, int e) {
  const int NCB = D / 32 + 1, FB = F / 32, NT = FB * NCB;
  if (e >= NT * 1024) return;
  const int ti = e >> 10, x = (e >> 6) & 15, lane = e & 63, r = lane & 31, g = lane >> 5;
  // eight chunks per step so that their loads are in flight together; fixed order of additions
  float sum = 0.f;
  const float *src = part + (int64_t)bh * n_chunks * NT * 1024 + e;
  int c = 0;
  for (; c + 8 <= n_chunks; c += 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = src[(int64_t)(c + i) * NT * 1024];
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += v[i];
  }
  for (; c + 4 <= n_chunks; c += 4) {
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = src[(int64_t)(c + i) * NT * 1024];
#pragma unroll
    for (int i = 0; i < 4; ++i) sum += v[i];
  }
  for (; c < n_chunks; ++c) sum += src[(int64_t)c * NT * 1024];
  const int fb = ti / NCB, cb = ti % NCB;
  const int ch = 32 * fb + crow(x, g);
  if (cb < D / 32) {
    const int dcol = 32 * cb + r;
    S[((int64_t)bh * F + ch) * D + dcol] = sum;
    const __bf16 hi = static_cast<__bf16>(sum);
    const __bf16 lo = static_cast<__bf16>(sum - static_cast<float>(hi));
    // inverse of the chained slot order: channel offset within its 32-block -> (s, g', t)
    const int cc = ch & 31, s = cc >> 4, w16 = cc & 15, g2 = (w16 >> 2) & 1, t = 4 * (w16 >> 3) + (w16 & 3);
    const int64_t idx = ((((int64_t)bh * (D / 32) + cb) * FB + fb) * 2 + s) * 512 + (g2 * 32 + r) * 8 + t;
    st_hi[idx] = hi;
    st_lo[idx] = lo;
  } else if (r == 0) {
    z[(int64_t)bh * F + ch] = sum;
  }
}

__global__ __launch_bounds__(256) void state_reduce_kernel(const float *__restrict__ part, float *__restrict__ S,
                                                           float *__restrict__ z, __bf16 *__restrict__ st_hi,
                                                           __bf16 *__restrict__ st_lo, int D, int F, int n_chunks) {
  state_reduce_body(part, S, z, st_hi, st_lo, D, F, n_chunks, blockIdx.y, blockIdx.x * 256 + threadIdx.x);
}

// The state reduction and the re-ordering of the query-side weights in one launch (two small, independent jobs that
// would otherwise each wait for the previous kernel to drain): rows y < BH of the grid reduce, rows BH + h prepare
// the weights of head h.
template <bool F32>
__global__ __launch_bounds__(256) void state_reduce_prep_kernel(const float *__restrict__ part, float *__restrict__ S,
                                                                float *__restrict__ z, __bf16 *__restrict__ st_hi,
                                                                __bf16 *__restrict__ st_lo, int D, int F, int n_chunks, int BH,
                                                                const void *__restrict__ w1, const void *__restrict__ w2,
                                                                __bf16 *__restrict__ w1f, __bf16 *__restrict__ w2f, int HD) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if ((int)blockIdx.y < BH) state_reduce_body(part, S, z, st_hi, st_lo, D, F, n_chunks, blockIdx.y, e);
  else weight_prep_body<F32>(w1, w2, w1f, w2f, D, HD, F, blockIdx.y - BH, e);
}

// ------------------------------------------------------------------------------------------------
// state_prefix_kernel (chunk-causal variant): grid as state_reduce_kernel.  Running sum of the chunk partials in
// chunk order; after every nsub of them (one causal chunk) the sum so far is written as that chunk's z and S^T
// fragments: st[bh][cc][...], z[bh][cc][F].  S (fp32) receives the total.
__global__ __launch_bounds__(256) void state_prefix_kernel(const float *__restrict__ part, float *__restrict__ S,
                                                           float *__restrict__ z, __bf16 *__restrict__ st_hi,
                                                           __bf16 *__restrict__ st_lo, int D, int F, int n_cc, int nsub) {
  const int NCB = D / 32 + 1, FB = F / 32, NT = FB * NCB;
  const int bh = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= NT * 1024) return;
  const int ti = e >> 10, x = (e >> 6) & 15, lane = e & 63, r = lane & 31, g = lane >> 5;
  const int fb = ti / NCB, cb = ti % NCB;
  const int ch = 32 * fb + crow(x, g);
  const float *src = part + (int64_t)bh * n_cc * nsub * NT * 1024 + e;
  float sum = 0.f;
  for (int cc = 0; cc < n_cc; ++cc) {
    for (int s = 0; s < nsub; ++s) sum += src[(int64_t)(cc * nsub + s) * NT * 1024];
    const int64_t sbh = (int64_t)bh * n_cc + cc;
    if (cb < D / 32) {
      const __bf16 hi = static_cast<__bf16>(sum);
      const __bf16 lo = static_cast<__bf16>(sum - static_cast<float>(hi));
      const int c5 = ch & 31, s = c5 >> 4, w16 = c5 & 15, g2 = (w16 >> 2) & 1, t = 4 * (w16 >> 3) + (w16 & 3);
      const int64_t idx = (((sbh * (D / 32) + cb) * FB + fb) * 2 + s) * 512 + (g2 * 32 + r) * 8 + t;
      st_hi[idx] = hi;
      st_lo[idx] = lo;
    } else if (r == 0) {
      z[sbh * F + ch] = sum;
    }
  }
  if (cb < D / 32) S[((int64_t)bh * F + ch) * D + 32 * cb + r] = sum;
}

// ------------------------------------------------------------------------------------------------
// state_window_kernel (local-window variant): grid as state_reduce_kernel; one chunk partial per query tile.  For
// tile t the state of the tokens OUTSIDE its window, i.e. the chunks before t - w and after t + w: a prefix that
// grows and a suffix that shrinks as t advances (no subtraction of nearly equal totals).  Output as in
// state_prefix_kernel: st[bh][t][...], z[bh][t][F].
__global__ __launch_bounds__(256) void state_window_kernel(const float *__restrict__ part, float *__restrict__ z,
                                                           __bf16 *__restrict__ st_hi, __bf16 *__restrict__ st_lo, int D,
                                                           int F, int n_t, int w) {
  const int NCB = D / 32 + 1, FB = F / 32, NT = FB * NCB;
  const int bh = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= NT * 1024) return;
  const int ti = e >> 10, x = (e >> 6) & 15, lane = e & 63, r = lane & 31, g = lane >> 5;
  const int fb = ti / NCB, cb = ti % NCB;
  const int ch = 32 * fb + crow(x, g);
  const float *src = part + (int64_t)bh * n_t * NT * 1024 + e;
  const int64_t cs = (int64_t)NT * 1024;
  float pre = 0.f, suf = 0.f;
  // chunks after the window of tile 0, four loads in flight at a time, added in a fixed order
  for (int c = n_t - 1; c > w; c -= 4) {
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = c - i > w ? src[(c - i) * cs] : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) suf += v[i];
  }
  const int c5 = ch & 31, s = c5 >> 4, w16 = c5 & 15, g2 = (w16 >> 2) & 1, tt = 4 * (w16 >> 3) + (w16 & 3);
  for (int t0 = 0; t0 < n_t; t0 += 4) {
    // tile t -> t + 1: chunk t - w leaves the window on the left, chunk t + 1 + w enters it on the right
    float leave[4], enter[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = t0 + i;
      leave[i] = (t - w >= 0 && t < n_t) ? src[(t - w) * cs] : 0.f;
      enter[i] = (t + 1 + w < n_t) ? src[(t + 1 + w) * cs] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = t0 + i;
      if (t < n_t) {
        const float sum = pre + suf;
        const int64_t sbh = (int64_t)bh * n_t + t;
        if (cb < D / 32) {
          const __bf16 hi = static_cast<__bf16>(sum);
          const __bf16 lo = static_cast<__bf16>(sum - static_cast<float>(hi));
          const int64_t idx = (((sbh * (D / 32) + cb) * FB + fb) * 2 + s) * 512 + (g2 * 32 + r) * 8 + tt;
          st_hi[idx] = hi;
          st_lo[idx] = lo;
        } else if (r == 0) {
          z[sbh * F + ch] = sum;
        }
        pre += leave[i];
        suf -= enter[i];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// host launchers

template <typename T>
static inline T *ws_ptr(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }

hipError_t launch_weight_prep(const Plan &pl, const ha_feature_map &fm, bool is_query, void *ws, hipStream_t st) {
  const int n = (pl.HD * pl.D > pl.F * pl.HD) ? pl.HD * pl.D : pl.F * pl.HD;
  dim3 grid((n + 255) / 256, pl.H);
  __bf16 *w1f = ws_ptr<__bf16>(ws, is_query ? pl.off_w1q : pl.off_w1k);
  __bf16 *w2f = ws_ptr<__bf16>(ws, is_query ? pl.off_w2q : pl.off_w2k);
  if (pl.f32) weight_prep_kernel<true><<<grid, 256, 0, st>>>(fm.w1, fm.w2, w1f, w2f, pl.D, pl.HD, pl.F);
  else weight_prep_kernel<false><<<grid, 256, 0, st>>>(fm.w1, fm.w2, w1f, w2f, pl.D, pl.HD, pl.F);
  return hipGetLastError();
}

hipError_t launch_compact(const Plan &pl, const void *k, const void *v, void *ws, hipStream_t st) {
  dim3 grid(pl.n_kblocks, pl.B * pl.H);
  bf16x8 *ksf = ws_ptr<bf16x8>(ws, pl.off_ks), *vsf = ws_ptr<bf16x8>(ws, pl.off_vs);
#define HA_COMPACT(DD, FF) \
  compact_kernel<DD, FF><<<grid, 256, 0, st>>>(k, v, ksf, vsf, pl.H, pl.NS, pl.LW > 0 ? 1 : pl.R, pl.G, pl.n_kblocks, pl.sb, \
                                               pl.sh, pl.sn)
  if (pl.D == 64) { if (pl.f32) HA_COMPACT(64, true); else HA_COMPACT(64, false); }
  else { if (pl.f32) HA_COMPACT(128, true); else HA_COMPACT(128, false); }
#undef HA_COMPACT
  return hipGetLastError();
}

hipError_t launch_state(const Plan &pl, const void *k, const void *v, const ha_feature_map &fm, void *ws,
                        hipStream_t st) {
  if (state_uses_pipelined_kernel(pl)) return launch_state_pipelined(pl, k, v, fm, ws, st);   // ha_state.hip
  dim3 grid(pl.n_chunks, pl.B * pl.H);
  const bf16x8 *w1f = ws_ptr<bf16x8>(ws, pl.off_w1k), *w2f = ws_ptr<bf16x8>(ws, pl.off_w2k);
  float *part = ws_ptr<float>(ws, pl.off_part);
#define HA_STATE(DD, HH, FF, F32) \
  state_kernel<DD, HH, FF, F32><<<grid, 256, 0, st>>>(k, v, w1f, w2f, fm.b1, fm.b2, part, pl.H, pl.NL, pl.R, pl.G, pl.CH, \
                                                     pl.P, pl.act_k, pl.sb, pl.sh, pl.sn, nullptr, nullptr, pl.N, pl.CC, pl.nsub)
  if (pl.D == 64) { if (pl.f32) HA_STATE(64, 64, 64, true); else HA_STATE(64, 64, 64, false); }
  else if (pl.HD == 128) { if (pl.f32) HA_STATE(128, 128, 128, true); else HA_STATE(128, 128, 128, false); }
  else { if (pl.f32) HA_STATE(128, 256, 256, true); else HA_STATE(128, 256, 256, false); }
#undef HA_STATE
  return hipGetLastError();
}

// The weighted pass over all N query tokens (value-distillation gradient): partial tiles of [dS | dz] to `part`.
hipError_t launch_weighted_state(const Plan &pl, const void *q, const void *gsign, const float *rs, const float *wp,
                                 const ha_feature_map &fm, const void *w1f_, const void *w2f_, float *part, int CH,
                                 int n_chunks, hipStream_t st) {
  if (state_uses_pipelined_kernel(pl))
    return launch_state_pipelined_weighted(pl, q, gsign, rs, wp, fm, w1f_, w2f_, part, CH, n_chunks, st);
  dim3 grid(n_chunks, pl.B * pl.H);
  const bf16x8 *w1f = static_cast<const bf16x8 *>(w1f_), *w2f = static_cast<const bf16x8 *>(w2f_);
#define HA_WSTATE(DD, F32) \
  state_kernel<DD, DD, DD, F32, true><<<grid, 256, 0, st>>>(q, gsign, w1f, w2f, fm.b1, fm.b2, part, pl.H, pl.N, 0, 1, CH, pl.P, \
                                                            pl.act_q, pl.sb, pl.sh, pl.sn, rs, wp)
  if (pl.D == 64) { if (pl.f32) HA_WSTATE(64, true); else HA_WSTATE(64, false); }
  else { if (pl.f32) HA_WSTATE(128, true); else HA_WSTATE(128, false); }
#undef HA_WSTATE
  return hipGetLastError();
}

hipError_t launch_state_reduce_with_prep(const Plan &pl, const ha_feature_map &phi_q, void *ws, hipStream_t st) {
  const int n_prep = ((pl.HD * pl.D > pl.F * pl.HD ? pl.HD * pl.D : pl.F * pl.HD) + 255) / 256;
  const int n_red = pl.n_state_tiles * 1024 / 256;
  dim3 grid(n_red > n_prep ? n_red : n_prep, pl.B * pl.H + pl.H);
#define HA_RP(F32) \
  state_reduce_prep_kernel<F32><<<grid, 256, 0, st>>>(ws_ptr<float>(ws, pl.off_part), ws_ptr<float>(ws, pl.off_S), \
      ws_ptr<float>(ws, pl.off_z), ws_ptr<__bf16>(ws, pl.off_sthi), ws_ptr<__bf16>(ws, pl.off_stlo), pl.D, pl.F, pl.n_chunks, \
      pl.B * pl.H, phi_q.w1, phi_q.w2, ws_ptr<__bf16>(ws, pl.off_w1q), ws_ptr<__bf16>(ws, pl.off_w2q), pl.HD)
  if (pl.f32) HA_RP(true); else HA_RP(false);
#undef HA_RP
  return hipGetLastError();
}

hipError_t launch_state_reduce(const Plan &pl, void *ws, hipStream_t st) {
  dim3 grid(pl.n_state_tiles * 1024 / 256, pl.B * pl.H);
  if (pl.LW > 0) {
    state_window_kernel<<<grid, 256, 0, st>>>(ws_ptr<float>(ws, pl.off_part), ws_ptr<float>(ws, pl.off_z),
                                              ws_ptr<__bf16>(ws, pl.off_sthi), ws_ptr<__bf16>(ws, pl.off_stlo), pl.D, pl.F,
                                              pl.n_cc, pl.LW / pl.CC);
    return hipGetLastError();
  }
  if (pl.CC > 0) {
    state_prefix_kernel<<<grid, 256, 0, st>>>(ws_ptr<float>(ws, pl.off_part), ws_ptr<float>(ws, pl.off_S),
                                              ws_ptr<float>(ws, pl.off_z), ws_ptr<__bf16>(ws, pl.off_sthi),
                                              ws_ptr<__bf16>(ws, pl.off_stlo), pl.D, pl.F, pl.n_cc, pl.nsub);
    return hipGetLastError();
  }
  state_reduce_kernel<<<grid, 256, 0, st>>>(ws_ptr<float>(ws, pl.off_part), ws_ptr<float>(ws, pl.off_S),
                                            ws_ptr<float>(ws, pl.off_z), ws_ptr<__bf16>(ws, pl.off_sthi),
                                            ws_ptr<__bf16>(ws, pl.off_stlo), pl.D, pl.F, pl.n_chunks);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Value-distillation loss (Sec. 3.3, Eq. "vd_loss"): sum |y - y_hat| over two [B, H, N, d] tensors.
// l1_partial_kernel: grid (L1_PARTS, B*H), 256 threads; workgroup (part, bh) walks a contiguous range of
// rows in 16-byte pieces, each thread adds its absolute differences in fp32 (a few hundred terms), the
// workgroup total is formed in fp64 in a fixed order.  l1_final_kernel adds the partials of every
// (batch, head) in part order, then the (batch, head) totals in order: bitwise reproducible.
constexpr int L1_PARTS = kL1Parts;

template <bool F32>
__global__ __launch_bounds__(256) void l1_partial_kernel(const void *__restrict__ ya, const void *__restrict__ yb,
                                                         double *__restrict__ partial, int H, int N, int D,
                                                         int64_t sb, int64_t sh, int64_t sn) {
  constexpr int EPP = F32 ? 4 : 8;                    // elements per 16-byte piece
  const int part = blockIdx.x, bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)(bh % H) * sh;
  const int rows_per = (N + L1_PARTS - 1) / L1_PARTS;
  const int r0 = part * rows_per, r1 = min(r0 + rows_per, N);
  const int ppr = D / EPP;                            // pieces per row
  float acc = 0.f;
  for (int i = threadIdx.x; i < (r1 - r0) * ppr; i += 256) {
    const int64_t off = base + (int64_t)(r0 + i / ppr) * sn + (i % ppr) * EPP;
    if constexpr (F32) {
      const f32x4 a = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(ya) + off);
      const f32x4 b = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(yb) + off);
#pragma unroll
      for (int t = 0; t < 4; ++t) acc += fabsf(a[t] - b[t]);
    } else {
      const bf16x8 a = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(ya) + off);
      const bf16x8 b = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(yb) + off);
#pragma unroll
      for (int t = 0; t < 8; ++t) acc += fabsf(static_cast<float>(a[t]) - static_cast<float>(b[t]));
    }
  }
  __shared__ double red[256];
  red[threadIdx.x] = (double)acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[(int64_t)bh * L1_PARTS + part] = red[0];
}

// loss[0] = total, loss[1 + bh] = per (batch, head)
__global__ __launch_bounds__(64) void l1_final_kernel(const double *__restrict__ partial, double *__restrict__ loss, int BH) {
  __shared__ double tot[64];
  double grand = 0.0;
  for (int b0 = 0; b0 < BH; b0 += 64) {
    const int bh = b0 + threadIdx.x;
    double s = 0.0;
    if (bh < BH) {
      for (int p = 0; p < L1_PARTS; ++p) s += partial[(int64_t)bh * L1_PARTS + p];
      loss[1 + bh] = s;
    }
    tot[threadIdx.x] = bh < BH ? s : 0.0;
    __syncthreads();
    if (threadIdx.x == 0)
      for (int i = 0; i < 64; ++i) grand += tot[i];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = grand;
}

size_t l1_partial_bytes(const Plan &pl) { return (size_t)pl.B * pl.H * L1_PARTS * sizeof(double); }

hipError_t launch_l1_distance(const Plan &pl, const void *ya, const void *yb, double *partial, double *loss,
                              hipStream_t st) {
  dim3 grid(L1_PARTS, pl.B * pl.H);
  if (pl.f32) l1_partial_kernel<true><<<grid, 256, 0, st>>>(ya, yb, partial, pl.H, pl.N, pl.D, pl.sb, pl.sh, pl.sn);
  else l1_partial_kernel<false><<<grid, 256, 0, st>>>(ya, yb, partial, pl.H, pl.N, pl.D, pl.sb, pl.sh, pl.sn);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_l1_final(pl, partial, loss, st);
}

hipError_t launch_l1_final(const Plan &pl, const double *partial, double *loss, hipStream_t st) {
  l1_final_kernel<<<1, 64, 0, st>>>(partial, loss, pl.B * pl.H);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Measurement aid, not a step of the method: nothing but dense bf16 32x32x16 matrix instructions on
// register operands (four independent accumulators per wave, eight waves per workgroup, one workgroup
// per compute unit).  Timed by a caller, it gives the matrix-core rate this device sustains, which
// depends on the operand values: all-zero operands toggle few wires and keep the clock at its
// ceiling, pseudo-random ones draw more power and the clock drops.
__global__ __launch_bounds__(512, 1) void mfma_probe_kernel(float *sink, int iters, int random_operands) {
  const unsigned tid = threadIdx.x + blockIdx.x * 512u;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      // integer hash -> value in [-1, 1) with a full 8-bit bf16 significand
      unsigned ha_ = (tid * 8u + i * 64u + t) * 2654435761u, hb_ = ha_ ^ 0x9e3779b9u;
      ha_ ^= ha_ >> 15; ha_ *= 2246822519u; ha_ ^= ha_ >> 13;
      hb_ ^= hb_ >> 15; hb_ *= 3266489917u; hb_ ^= hb_ >> 13;
      const float fa = random_operands ? (float)(int)(ha_ >> 16) * (1.0f / 32768.0f) - 1.0f : 0.0f;
      const float fb = random_operands ? (float)(int)(hb_ >> 16) * (1.0f / 32768.0f) - 1.0f : 0.0f;
      a[i][t] = static_cast<__bf16>(fa);
      b[i][t] = static_cast<__bf16>(fb);
    }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = mfma32(a[(i + u) & 3], b[i], acc[i]);
  }
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) r += acc[i][v];
  sink[tid] = r;
}

hipError_t launch_mfma_probe(float *sink, int workgroups, int iters, int random_operands, hipStream_t st) {
  mfma_probe_kernel<<<workgroups, 512, 0, st>>>(sink, iters, random_operands);
  return hipGetLastError();
}

}  // namespace ha
