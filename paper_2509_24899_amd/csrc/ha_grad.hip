// Gradient of the value-distillation loss (Attention Surgery, Sec. 3.3: Eq. "vd_loss" and the update line of
// Alg. "distil") with respect to the two feature maps, gfx950.  q, k, v are constants of the isolated layer.
//
// With y_hat_i = num_i / den_i, num_i = a_i + phi_q(q_i) S, den_i = l_i + phi_q(q_i).z (Eq. "hybrid") and
// g_i = sign(y_hat_i - y_i):
//     dnum_i = g_i / den_i,   dden_i = -(g_i . y_hat_i) / den_i
//     dphi_q(q_i) = S dnum_i + dden_i z          dS = sum_i phi_q(q_i)^T dnum_i,   dz = sum_i dden_i phi_q(q_i)
//     dphi_k(k_j) = dS v_j + dz   (j in T_L)
// and each dphi goes back through  phi = t^p (slice powers), t = softmax / exp / relu (u), u = W2 h + b2,
// h = relu(W1 x + b1)  to  dW2 = sum du h^T, db2 = sum du, dW1 = sum dpre x^T, db1 = sum dpre.
//
//   grad_weight_prep_kernel   W2^T as A-operand fragments in chained order (for dh = W2^T du)
//   natural_frags_kernel      an fp32 matrix (S or dS) as hi + lo bf16 A-operand fragments in natural order
//   vd_rows_kernel            per row: the sign tensor g (bf16), 1 / den_i and -(g_i . y_hat_i)
//   (state_kernel, weighted)  [dS | dz] over all query tokens: the forward's state pass with q in place of k, the
//                             sign tensor in place of v, rows scaled by 1 / den_i and dden_i den_i in place of 1
//   grad_kernel<QUERY>        one pass over the query tokens (QUERY) or the linear key tokens: recomputes the
//                             map, forms dphi, du, dpre per 32-token column block in registers and contracts
//                             over the tokens through LDS into per-chunk partial tiles of [dW2 | db2], [dW1 | db1]
//   grad_reduce_kernel        fixed-order sum of the partial tiles over chunks (and over the batch for the
//                             shared parameters) into plain row-major fp32
//
// As in the forward, every product is computed transposed (channels x tokens): one lane owns one token.
#include "ha_device.h"
#include "ha_mlp128.h"
#include "ha_plan.h"

namespace ha {

// ------------------------------------------------------------------------------------------------
// grad_weight_prep_kernel: grid (ceil(HD*F / 256), H)
//   w2tf[h][hb][fb][s][lane][t] = W2[h][32fb + crow(8s + t, g)][32hb + r]
template <bool F32>
static __device__ __forceinline__ void grad_weight_prep_body(const void *__restrict__ w2, __bf16 *__restrict__ w2tf, int HD,
                                                             int F, int h, int e) {
  if (e >= HD * F) return;
  const int t = e & 7, lane = (e >> 3) & 63, rest = e >> 9;
  const int r = lane & 31, g = lane >> 5;
  const int FB = F / 32;
  const int s = rest & 1, fb = (rest >> 1) % FB, hb = (rest >> 1) / FB;
  const int64_t src = ((int64_t)h * F + 32 * fb + crow(8 * s + t, g)) * HD + 32 * hb + r;
  float val;
  if constexpr (F32) val = static_cast<const float *>(w2)[src];
  else val = static_cast<float>(static_cast<const __bf16 *>(w2)[src]);
  w2tf[(int64_t)h * HD * F + e] = static_cast<__bf16>(val);
}
template <bool F32>
__global__ __launch_bounds__(256) void grad_weight_prep_kernel(const void *__restrict__ w2, __bf16 *__restrict__ w2tf,
                                                               int HD, int F) {
  grad_weight_prep_body<F32>(w2, w2tf, HD, F, blockIdx.y, blockIdx.x * 256 + threadIdx.x);
}

// natural_frags_kernel: grid (ceil(rows*cols / 256), n_mat)
//   hi/lo[m][rb][ks][lane][t] = M[m][32rb + r][16ks + 8g + t]
static __device__ __forceinline__ void natural_frags_body(const float *__restrict__ M, __bf16 *__restrict__ hi,
                                                          __bf16 *__restrict__ lo, int rows, int cols, int m, int e) {
  if (e >= rows * cols) return;
  const int t = e & 7, lane = (e >> 3) & 63, rest = e >> 9;
  const int r = lane & 31, g = lane >> 5;
  const int KS = cols / 16;
  const int ks = rest % KS, rb = rest / KS;
  const float val = M[((int64_t)m * rows + 32 * rb + r) * cols + 16 * ks + 8 * g + t];
  const __bf16 h = static_cast<__bf16>(val);
  hi[(int64_t)m * rows * cols + e] = h;
  lo[(int64_t)m * rows * cols + e] = static_cast<__bf16>(val - static_cast<float>(h));
}
__global__ __launch_bounds__(256) void natural_frags_kernel(const float *__restrict__ M, __bf16 *__restrict__ hi,
                                                            __bf16 *__restrict__ lo, int rows, int cols) {
  natural_frags_body(M, hi, lo, rows, cols, blockIdx.y, blockIdx.x * 256 + threadIdx.x);
}

// grad_operands_kernel: the five small jobs ahead of the gradient passes of the square maps (d -> d -> d) in one
// launch, grid (ceil(D*D / 256), 4 H + B*H): rows [0, H) and [H, 2 H) the forward fragments of phi_q's and phi_k's
// weights, [2 H, 3 H) and [3 H, 4 H) their W2^T fragments, the rest S as hi + lo natural-order fragments.
struct GradOperands {
  const void *w1q, *w2q, *w1k, *w2k;
  __bf16 *w1qf, *w2qf, *w1kf, *w2kf, *w2tq, *w2tk;
  const float *S;
  __bf16 *s_hi, *s_lo;
  int D, H;
};
template <bool F32>
__global__ __launch_bounds__(256) void grad_operands_kernel(GradOperands o) {
  const int e = blockIdx.x * 256 + threadIdx.x, y = blockIdx.y, D = o.D, H = o.H;
  if (y < H) weight_prep_body<F32>(o.w1q, o.w2q, o.w1qf, o.w2qf, D, D, D, y, e);
  else if (y < 2 * H) weight_prep_body<F32>(o.w1k, o.w2k, o.w1kf, o.w2kf, D, D, D, y - H, e);
  else if (y < 3 * H) grad_weight_prep_body<F32>(o.w2q, o.w2tq, D, D, y - 2 * H, e);
  else if (y < 4 * H) grad_weight_prep_body<F32>(o.w2k, o.w2tk, D, D, y - 3 * H, e);
  else natural_frags_body(o.S, o.s_hi, o.s_lo, D, D, y - 4 * H, e);
}

// ------------------------------------------------------------------------------------------------
// vd_rows_kernel: grid (ceil(N / rows_per_block), B*H), 256 threads, D / 8 threads per row.
//   gsign[bh][i][:] = sign(y_hat_i - y_i) (bf16, dense),  rs[bh][i] = 1 / den_i,  wp[bh][i] = -(g_i . y_hat_i)
template <int D, bool F32>
__global__ __launch_bounds__(256) void vd_rows_kernel(const void *__restrict__ y_teacher, const void *__restrict__ y_student,
                                                      const float *__restrict__ row_den, bf16x8 *__restrict__ gsign,
                                                      float *__restrict__ rs, float *__restrict__ wp, int H, int N,
                                                      int64_t sb, int64_t sh, int64_t sn) {
  constexpr int TPR = D / 8, RPB = 256 / TPR;
  const int bh = blockIdx.y;
  const int row = blockIdx.x * RPB + threadIdx.x / TPR, c8 = threadIdx.x % TPR;
  const bool valid = row < N;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)(bh % H) * sh + (int64_t)(valid ? row : 0) * sn + c8 * 8;
  float yt[8], ys[8];
  if constexpr (F32) {
    const float *a = static_cast<const float *>(y_teacher) + base, *b = static_cast<const float *>(y_student) + base;
#pragma unroll
    for (int t = 0; t < 8; ++t) { yt[t] = a[t]; ys[t] = b[t]; }
  } else {
    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(y_teacher) + base);
    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(y_student) + base);
#pragma unroll
    for (int t = 0; t < 8; ++t) { yt[t] = static_cast<float>(a[t]); ys[t] = static_cast<float>(b[t]); }
  }
  bf16x8 gs;
  float dot = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const float diff = ys[t] - yt[t];
    const float sg = diff > 0.f ? 1.f : (diff < 0.f ? -1.f : 0.f);
    gs[t] = static_cast<__bf16>(sg);
    dot += sg * ys[t];
  }
#pragma unroll
  for (int m = 1; m < TPR; m <<= 1) dot += __shfl_xor(dot, m);
  if (valid) {
    gsign[((int64_t)bh * N + row) * TPR + c8] = gs;
    if (c8 == 0) {
      rs[(int64_t)bh * N + row] = 1.0f / row_den[(int64_t)bh * N + row];
      wp[(int64_t)bh * N + row] = -dot;
    }
  }
}

// vd_rows_loss_kernel (bf16 io): what vd_rows_kernel writes, and in the same pass over the two outputs the partial
// sums of || y - y_hat ||_1 exactly as l1_partial_kernel forms them (same grid (parts, B*H), same walk of a
// contiguous range of rows in 16-byte pieces, same order of the additions), so the loss is the same number bit for
// bit and the two tensors are read once instead of twice.
template <int D>
__global__ __launch_bounds__(256) void vd_rows_loss_kernel(const void *__restrict__ y_teacher, const void *__restrict__ y_student,
                                                           const float *__restrict__ row_den, bf16x8 *__restrict__ gsign,
                                                           float *__restrict__ rs, float *__restrict__ wp,
                                                           double *__restrict__ partial, int H, int N, int64_t sb, int64_t sh,
                                                           int64_t sn) {
  constexpr int TPR = D / 8;                          // 16-byte pieces (threads) per row; 256 is a multiple of it
  const int part = blockIdx.x, bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)(bh % H) * sh;
  const int rows_per = (N + kL1Parts - 1) / kL1Parts;
  const int r0 = part * rows_per, r1 = min(r0 + rows_per, N);
  const int n_pieces = max(r1 - r0, 0) * TPR;
  float acc = 0.f;
  // every thread of a row group runs the same number of trips, so that the exchange below is among live lanes
  for (int i0 = 0; i0 < n_pieces; i0 += 256) {
    const int i = i0 + threadIdx.x;
    const bool valid = i < n_pieces;
    const int row = r0 + (valid ? i / TPR : 0), c8 = i % TPR;
    const int64_t off = base + (int64_t)row * sn + c8 * 8;
    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(y_teacher) + off);
    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(y_student) + off);
    bf16x8 gs;
    float dot = 0.f, ad[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float yt = static_cast<float>(a[t]), ys = static_cast<float>(b[t]);
      const float diff = ys - yt;
      const float sg = diff > 0.f ? 1.f : (diff < 0.f ? -1.f : 0.f);
      gs[t] = static_cast<__bf16>(sg);
      dot += sg * ys;
      ad[t] = fabsf(yt - ys);
    }
#pragma unroll
    for (int m = 1; m < TPR; m <<= 1) dot += __shfl_xor(dot, m);
    if (valid) {
#pragma unroll
      for (int t = 0; t < 8; ++t) acc += ad[t];          // (one term at a time, as the loss kernel adds them)
      gsign[((int64_t)bh * N + row) * TPR + c8] = gs;
      if (c8 == 0) {
        rs[(int64_t)bh * N + row] = 1.0f / row_den[(int64_t)bh * N + row];
        wp[(int64_t)bh * N + row] = -dot;
      }
    }
  }
  __shared__ double red[256];
  red[threadIdx.x] = (double)acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[(int64_t)bh * kL1Parts + part] = red[0];
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// ------------------------------------------------------------------------------------------------
// grad_kernel: grid (n_chunks, B*H), 4 waves; square maps (hidden width = feature width = D).  A chunk is CH
// tokens of the pass's token set, walked in tiles of 128; wave w owns tokens 32 w .. 32 w + 31 of a tile.
//
// Per tile and wave, in registers (lane = token, registers = channels, as in the forward):
//   h, t = activation(W2 h + b2)                       recomputed
//   dphi = rs (M u) + wz zvec                          M = S, u = g_i, rs = 1/den_i, wz = dden_i   (queries)
//                                                      M = dS, u = v_j, rs = wz = 1                 (keys)
//   du   = activation'(t) (dphi p t^(p-1)),  dpre = (W2^T du) [h > 0]
// then two contractions over the 128 tokens of the tile, each through the same two LDS arrays
// (A side: rows x tokens, B side: columns x tokens, tokens contiguous, swizzled as in the state pass):
//   [dW2 | db2] += du [h | 1]^T
//   [dW1 | db1] += dpre [x | 1]^T
// Output row block w of each product belongs to wave w (waves >= T idle during the contractions).
// Partial tiles go to part[bh][chunk][set][tile][v][lane], set order: dW2, dW1.
// t^e for a small wave-uniform exponent e in 0..7, branch-free
static __device__ __forceinline__ float pow_small(float t, int e) {
  const float t2 = t * t;
  float r = (e & 1) ? t : 1.f;
  r = (e & 2) ? r * t2 : r;
  r = (e & 4) ? r * (t2 * t2) : r;
  return r;
}

struct GradArgs {
  const void *x;                    // q (queries) or k (keys): io dtype, strided
  const void *u;                    // queries: sign tensor, bf16 dense [B*H][N][D]; keys: v, io dtype, strided
  const float *rs, *wp;             // queries only: [B*H][N]
  const bf16x8 *w1f, *w2f, *w2tf;   // per head
  const float *b1, *b2;             // per head, may be null
  const bf16x8 *m_hi, *m_lo;        // [B*H][D*D/8]: natural-order fragments of S (queries) or dS (keys)
  const float *zvec;                // [B*H][D]: z (queries) or dz (keys)
  float *part;
  int H, N, NT, R, G, CH, P, act;
  int64_t sb, sh, sn;
};

template <int D, bool F32, bool QUERY>
__global__ __launch_bounds__(256, 1) void grad_kernel(GradArgs a) {
  constexpr int TOK = 128, PITCH = TOK + 8;
  constexpr int KS = D / 16, T = D / 32, NCB = T + 1, NT2 = T * NCB;
  constexpr int NSET = 2;
  __shared__ __align__(16) __bf16 ft[D][PITCH];
  __shared__ __align__(16) __bf16 vt[D][PITCH];
  __shared__ bf16x8 wlds[2 * D * D / 8];
  __shared__ float blds[3 * D];
  const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % a.H;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  {
    const bf16x8 *w1g = a.w1f + (int64_t)h * (D * D / 8), *w2g = a.w2f + (int64_t)h * (D * D / 8);
    for (int i = tid; i < D * D / 8; i += 256) {
      wlds[i] = w1g[i];
      wlds[D * D / 8 + i] = w2g[i];
    }
    for (int i = tid; i < D; i += 256) {
      blds[i] = a.b1 ? a.b1[(int64_t)h * D + i] : 0.f;
      blds[D + i] = a.b2 ? a.b2[(int64_t)h * D + i] : 0.f;
      blds[2 * D + i] = a.zvec[(int64_t)bh * D + i];
    }
    __syncthreads();
  }
  const lds_frag_ptr w1f = (lds_frag_ptr)&wlds[0], w2f = (lds_frag_ptr)&wlds[D * D / 8];
  const GlobalFrags w2tf = global_frags(a.w2tf + (int64_t)h * (D * D / 8), D * D * 2);
  const GlobalFrags mhi = global_frags(a.m_hi + (int64_t)bh * (D * D / 8), D * D * 2);
  const GlobalFrags mlo = global_frags(a.m_lo + (int64_t)bh * (D * D / 8), D * D * 2);
  const float *b1 = &blds[0], *b2 = &blds[D], *zl = &blds[2 * D];

  const LinearMap lmap(QUERY ? 0 : a.R, a.G);

  f32x16 acc2[NCB], acc1[NCB];
#pragma unroll
  for (int i = 0; i < NCB; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      acc2[i][x] = 0.f;
      acc1[i][x] = 0.f;
    }

  // LDS addressing (see the state pass): element (row, token) at row * PITCH + (((token / 8) ^ sw(row)) * 8 +
  // token % 8), sw(row) = ((row / 8) % 4) * 2
  // (the address pieces below are the same in every tile; they are formed from `zt`, a zero the compiler cannot
  // see through that is refreshed per tile, so that they are recomputed with two or three instructions where
  // they are used instead of living, i.e. being spilled, across the whole tile)
  const int tf = w * 32 + r;
  int zt = 0;
  __bf16 *ftp = &ft[0][0];
  __bf16 *vtp = &vt[0][0];
  auto park_chained = [&](__bf16 *arr, const bf16x8 (&val)[T][2]) {
    const int tfz = tf + zt;
    int fcol[4];                                          // chained-order writes: rows 32 b + 8 q + 4 g + e
#pragma unroll
    for (int q = 0; q < 4; ++q) fcol[q] = (4 * g) * PITCH + ((((tfz >> 3) ^ (2 * q)) << 3) | (tfz & 7));
#pragma unroll
    for (int b = 0; b < T; ++b)
#pragma unroll
      for (int x = 0; x < 16; ++x) arr[(32 * b + 8 * (x >> 2) + (x & 3)) * PITCH + fcol[x >> 2]] = val[b][x >> 3][x & 7];
  };
  auto park_natural = [&](__bf16 *arr, const bf16x8 (&val)[KS]) {   // rows 16 ks + 8 g + i
    const int tfz = tf + zt;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int sw = ((2 * ks + g) & 3) << 1;
      const int col = (((tfz >> 3) ^ sw) << 3) | (tfz & 7);
#pragma unroll
      for (int i = 0; i < 8; ++i) arr[(16 * ks + 8 * g + i) * PITCH + col] = val[ks][i];
    }
  };
  // row block w of (A side) x all column blocks of (B side), plus the extra column block
  auto contract = [&](f32x16 (&acc)[NCB]) {
    if (w < T) {
      const __bf16 one = static_cast<__bf16>(r == 0 ? 1.0f : 0.0f);
      const bf16x8 ones = bf16x8{one, one, one, one, one, one, one, one};
      const int rz = r + zt;
      const int rsw = ((rz >> 3) & 3) << 1;
      const int arow = (32 * w + rz) * PITCH, brow = rz * PITCH;
      // four 16-token slices at a time: their fragments are requested before the matrix instructions that use them
      constexpr int KB = 4;
#pragma unroll
      for (int ks0 = 0; ks0 < TOK / 16; ks0 += KB) {
        bf16x8 af[KB], bfr[KB][T];
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) {
          const int col = ((2 * (ks0 + kk) + g) ^ rsw) << 3;
          af[kk] = *reinterpret_cast<const bf16x8 *>(&ftp[arow + col]);
#pragma unroll
          for (int cb = 0; cb < T; ++cb) bfr[kk][cb] = *reinterpret_cast<const bf16x8 *>(&vtp[brow + 32 * cb * PITCH + col]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KB; ++kk)
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb) acc[cb] = mfma32(af[kk], cb < T ? bfr[kk][cb] : ones, acc[cb]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  const int t_begin = chunk * a.CH;
  const int t_end = min(t_begin + a.CH, a.NT);
  // the rows of the next tile are requested while the current one is still being contracted
  bf16x8 xf[KS], uf[KS];
  auto request_x = [&](int t0) {
    const int tok = lmap.token(min(t0 + tf, a.NT - 1));
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) xf[ks] = load8<F32>(a.x, base + (int64_t)tok * a.sn + 16 * ks + 8 * g);
  };
  auto request_u = [&](int t0) {
    const int tok = lmap.token(min(t0 + tf, a.NT - 1));
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if constexpr (QUERY) uf[ks] = static_cast<const bf16x8 *>(a.u)[((int64_t)bh * a.N + tok) * (D / 8) + 2 * ks + g];
      else uf[ks] = load8<F32>(a.u, base + (int64_t)tok * a.sn + 16 * ks + 8 * g);
    }
  };
  request_x(t_begin);
  request_u(t_begin);
  for (int t0 = t_begin; t0 < t_end; t0 += TOK) {
    const bool valid = t0 + tf < a.NT;
    const int tok = lmap.token(min(t0 + tf, a.NT - 1));
    // weights, biases and the fragments of M are the same in every tile: reading them through an offset the
    // compiler cannot see through keeps the reads in the loop (hoisted, they would fill the register file)
    const int z0 = opaque_zero();
    zt = z0;
    const lds_frag_ptr w1t = w1f + z0, w2t = w2f + z0;
    const float *b1t = b1 + z0, *b2t = b2 + z0, *zt = zl + z0;
    __builtin_assume(b1t != nullptr);
    __builtin_assume(b2t != nullptr);
    float rs_ = 1.f, wp_ = 1.f;
    if constexpr (QUERY) {
      rs_ = a.rs[(int64_t)bh * a.N + tok];
      wp_ = a.wp[(int64_t)bh * a.N + tok];
    }
    const float wz_ = QUERY ? wp_ * rs_ : 1.f;             // dden_i = -(g_i . y_hat_i) / den_i

    // the map, recomputed: h (hi + lo), t = positive output before the slice powers.  h goes to the B side
    // array right away; its ReLU gate is kept as one bit per hidden unit.
    f32x16 tt[T];
    unsigned gate[(T + 1) / 2];
    {
      bf16x8 h_hi[T][2], h_lo[T][2];
      feature_mlp_layer1<D, D, true>(xf, w1t, b1t, lane, g, h_hi, h_lo);
#pragma unroll
      for (int i = 0; i < (T + 1) / 2; ++i) gate[i] = 0u;
#pragma unroll
      for (int hb = 0; hb < T; ++hb)
#pragma unroll
        for (int x = 0; x < 16; ++x)
          gate[hb >> 1] |= (static_cast<float>(h_hi[hb][x >> 3][x & 7]) > 0.f ? 1u : 0u) << (16 * (hb & 1) + x);
      feature_mlp_layer2<D, D, true>(h_hi, h_lo, w2t, b2t, lane, g, tt);
      // consumed by the vector ALU from here on: keep the tiles out of the accumulator file, which the persistent
      // partial sums fill
#pragma unroll
      for (int fb = 0; fb < T; ++fb) asm volatile("" : "+v"(tt[fb]));
      feature_activation<T>(tt, g, a.act, 1, D);
      park_chained(vtp, h_hi);
    }
    // dphi = rs (M u) + wz zvec
    // (the fragments of M come from L2: the next half block (lo or hi part of one channel block, 8 fragments) is
    // requested before the chain of the current one starts, so that one round trip is exposed per tile instead
    // of one per instruction; larger batches cost more in spilled registers than they save)
    f32x16 dv[T];
    bf16x8 mf[2][KS];
    auto request_m = [&](int step, bf16x8 (&dst)[KS]) {       // step = 2 fb + (0: lo part, 1: hi part)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        dst[ks] = (step & 1) ? frag_at(mhi, (step >> 1) * KS + ks, lane, z0) : frag_at(mlo, (step >> 1) * KS + ks, lane, z0);
    };
    request_m(0, mf[0]);
#pragma unroll
    for (int fb = 0; fb < T; ++fb) {
      f32x16 acc;
#pragma unroll
      for (int x = 0; x < 16; ++x) acc[x] = 0.f;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int step = 2 * fb + half;
        if (step + 1 < 2 * T) request_m(step + 1, mf[(step + 1) & 1]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = mfma32(mf[step & 1][ks], uf[ks], acc);
      }
#pragma unroll
      for (int x = 0; x < 16; ++x) dv[fb][x] = rs_ * acc[x] + wz_ * zt[32 * fb + crow(x, g)];
    }

    __builtin_amdgcn_sched_barrier(0);
    request_u(t0 + TOK);
    __builtin_amdgcn_sched_barrier(0);
    // back through the slice powers and the activation: dv becomes du
    {
      float dot = 0.f;
#pragma unroll
      for (int fb = 0; fb < T; ++fb)
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const int extra = ((32 * fb + 8 * (x >> 2)) * a.P) / D;   // channel / Dp: slice power p = extra + 1 (wave-uniform)
          const float t0v = tt[fb][x];
          dv[fb][x] *= (float)(extra + 1) * pow_small(t0v, extra);   // d/dt of t^p
          dot += t0v * dv[fb][x];
        }
      if (a.act == 0) {
        dot = xhalf_sum(dot);
#pragma unroll
        for (int fb = 0; fb < T; ++fb)
#pragma unroll
          for (int x = 0; x < 16; ++x) dv[fb][x] = tt[fb][x] * (dv[fb][x] - dot);
      } else if (a.act == 1) {
#pragma unroll
        for (int fb = 0; fb < T; ++fb)
#pragma unroll
          for (int x = 0; x < 16; ++x) dv[fb][x] *= tt[fb][x];
      } else {
#pragma unroll
        for (int fb = 0; fb < T; ++fb)
#pragma unroll
          for (int x = 0; x < 16; ++x) dv[fb][x] = tt[fb][x] > 0.f ? dv[fb][x] : 0.f;
      }
    }
    bf16x8 dub[T][2];
#pragma unroll
    for (int fb = 0; fb < T; ++fb)
#pragma unroll
      for (int x = 0; x < 16; ++x) dub[fb][x >> 3][x & 7] = static_cast<__bf16>(valid ? dv[fb][x] : 0.f);

    // [dW2 | db2] += du [h | 1]^T
    park_chained(ftp, dub);
    __syncthreads();
    contract(acc2);
    // dpre = (W2^T du) [h > 0]   (registers only: overlaps the other waves' contraction)
    bf16x8 dpb[T][2];
    bf16x8 wt[2][2 * T];
    auto request_w = [&](int hb, bf16x8 (&dst)[2 * T]) {
#pragma unroll
      for (int i = 0; i < 2 * T; ++i) dst[i] = frag_at(w2tf, hb * T * 2 + i, lane, z0);
    };
    request_w(0, wt[0]);
#pragma unroll
    for (int hb = 0; hb < T; ++hb) {
      f32x16 acc;
#pragma unroll
      for (int x = 0; x < 16; ++x) acc[x] = 0.f;
      if (hb + 1 < T) request_w(hb + 1, wt[(hb + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int fb = 0; fb < T; ++fb)
#pragma unroll
        for (int s = 0; s < 2; ++s) acc = mfma32(wt[hb & 1][fb * 2 + s], dub[fb][s], acc);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int x = 0; x < 16; ++x)
        dpb[hb][x >> 3][x & 7] = static_cast<__bf16>((gate[hb >> 1] >> (16 * (hb & 1) + x)) & 1u ? acc[x] : 0.f);
    }
    __syncthreads();
    // [dW1 | db1] += dpre [x | 1]^T
    park_chained(ftp, dpb);
    park_natural(vtp, xf);
    __builtin_amdgcn_sched_barrier(0);
    request_x(t0 + TOK);
    __syncthreads();
    contract(acc1);
    __syncthreads();
  }
  if (w < T) {
    float *dst = a.part + (((int64_t)bh * gridDim.x + chunk) * NSET) * NT2 * 1024 + (int64_t)w * NCB * 1024;
#pragma unroll
    for (int i = 0; i < NCB; ++i)
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        dst[i * 1024 + x * 64 + lane] = acc2[i][x];
        dst[(NT2 + i) * 1024 + x * 64 + lane] = acc1[i][x];
      }
  }
}

// ------------------------------------------------------------------------------------------------
// grad_split_kernel: the pass of grad_kernel for d = 128 in two roles (the arrangement of the forward's state pass):
// grid (n_chunks, B*H), 8 waves, two per SIMD.
//   waves 0 - 3  per tile of 128 tokens, 32 token rows each, all in registers: the map recomputed, dphi, du; dpre.
//                Their operands for the two contractions leave as row-major bf16 tiles in LDS ([token][channel],
//                8-byte pieces of four consecutive channels, the C layout of the matrix instructions; x as 16-byte
//                pieces), 16-byte pieces XOR-swizzled over sixteen rows.
//   waves 4 - 7  own row block w of both partial sums, [dW2 | db2] += du [h | 1]^T and [dW1 | db1] += dpre [x | 1]^T,
//                and contract over the tokens with both operands read through the transposing LDS reads
//                (ds_read_b64_tr_b16), while the first four waves go on: W2^T du runs under the first contraction,
//                the next tile's map under the second.
// M (S or dS as hi + lo fragments, 64 KiB) passes through the same two tiles: the contraction waves fetch it
// (direct-to-LDS) once the tiles are free, the other waves read their fragments of it from LDS instead of each from
// L2.  W2^T sits in LDS for the whole workgroup (30 of its 32 fragments: that is what fits; the last two come from L2).
// Six barriers per tile: A1 (the second contraction of the tile before has read both tiles), M1 (M has landed), M2
// (its fragments have been read), B1 (h and du are in place), A2 (the first contraction has read them), B2 (dpre and x
// are in place).  Every wave of either role passes all six once per tile and both roles count the same tiles.
// Partial tiles as grad_kernel writes them.
// ACT0: the output activation of the map is the softmax over the channels.
template <bool F32, bool QUERY, bool ACT0>
__global__ __launch_bounds__(512, 1) void grad_split_kernel(GradArgs a) {
  constexpr int D = 128, TOK = 128, ROWB = 2 * D;
  constexpr int KS = D / 16, T = D / 32, NCB = T + 1, NT2 = T * NCB;
  constexpr int NSET = 2;
  __shared__ bf16x8 wlds[2 * D * D / 8];
  constexpr int W2T_LDS = 30;                        // fragments of W2^T that fit next to everything else (of 32)
  __shared__ bf16x8 w2t_lds[W2T_LDS * 64];
  __shared__ __align__(16) float blds[3 * D];
  __shared__ __align__(16) char a_t[TOK * ROWB];     // A side of a contraction: du, then dpre
  __shared__ __align__(16) char b_t[TOK * ROWB];     // B side: h, then x
  const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % a.H;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int w = wave & 3;
  {
    const bf16x8 *w1g = a.w1f + (int64_t)h * (D * D / 8), *w2g = a.w2f + (int64_t)h * (D * D / 8);
    const bf16x8 *w2tg = a.w2tf + (int64_t)h * (D * D / 8);
    for (int i = tid; i < D * D / 8; i += 512) {
      wlds[i] = w1g[i];
      wlds[D * D / 8 + i] = w2g[i];
      if (i < W2T_LDS * 64) w2t_lds[i] = w2tg[i];
    }
    for (int i = tid; i < D; i += 512) {
      blds[i] = a.b1 ? a.b1[(int64_t)h * D + i] : 0.f;
      blds[D + i] = a.b2 ? a.b2[(int64_t)h * D + i] : 0.f;
      blds[2 * D + i] = a.zvec[(int64_t)bh * D + i];
    }
  }
  const int t_begin = chunk * a.CH;
  const int t_end = min(t_begin + a.CH, a.NT);
  // piece p (16 bytes) of token row t sits at p ^ psw(t): the 32 rows one 8-byte write instruction touches fall on
  // sixteen different pieces, and a transposing read finds its four rows in four different 64-byte groups
  auto psw = [](int t) { return 4 * (t & 3) + ((t >> 2) & 3); };
  const LinearMap lmap(QUERY ? 0 : a.R, a.G);
  const int tf = w * 32 + r;                         // this lane's token row of a tile, in either role
  const int row_off = tf * ROWB, row_sw = psw(tf);
  auto request_x = [&](int t0, bf16x8 (&dst)[KS]) {
    const int tok = lmap.token(min(t0 + tf, a.NT - 1));
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) dst[ks] = load8<F32>(a.x, base + (int64_t)tok * a.sn + 16 * ks + 8 * g);
  };

  if (wave < 4) {
    // ============================== the map and its backward chain, 32 token rows per wave ==============================
    const lds_frag_ptr w1f = (lds_frag_ptr)&wlds[0], w2f = (lds_frag_ptr)&wlds[D * D / 8];
    const GlobalFrags w2tf = global_frags(a.w2tf + (int64_t)h * (D * D / 8), D * D * 2);
    const lds_frag_ptr w2tl = (lds_frag_ptr)&w2t_lds[0];
    const lds_frag_ptr mhi = (lds_frag_ptr)(const bf16x8 *)a_t, mlo = (lds_frag_ptr)(const bf16x8 *)b_t;   // M while it is staged
    const float *b1 = &blds[0], *b2 = &blds[D], *zl = &blds[2 * D];
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    // a [T][2] set of chained-order bf16 tiles (registers 4 q .. 4 q + 3 of tile fb: channels 32 fb + 8 q + 4 g .. + 3)
    // as 8-byte pieces of this lane's token row
    // (the addresses are formed where they are used, from a swizzle value the compiler cannot see through: kept across
    // the tile they would be spilled, and a reload costs more than the two instructions that make one)
    auto write_chained = [&](char *tile, const bf16x8 (&val)[T][2]) {
      const int sw_now = row_sw + opaque_zero();
#pragma unroll
      for (int fb = 0; fb < T; ++fb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const u32x4 t4 = __builtin_bit_cast(u32x4, val[fb][q >> 1]);
          const u32x2 four = {t4[2 * (q & 1)], t4[2 * (q & 1) + 1]};
          *reinterpret_cast<u32x2 *>(tile + row_off + 8 * g + (((4 * fb + q) ^ sw_now) << 4)) = four;
        }
    };
    bf16x8 xf[KS], uf[KS];
    auto request_u = [&](int t0) {
      const int tok = lmap.token(min(t0 + tf, a.NT - 1));
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if constexpr (QUERY) uf[ks] = static_cast<const bf16x8 *>(a.u)[((int64_t)bh * a.N + tok) * (D / 8) + 2 * ks + g];
        else uf[ks] = load8<F32>(a.u, base + (int64_t)tok * a.sn + 16 * ks + 8 * g);
      }
    };
    request_x(t_begin, xf);
    __syncthreads();                                  // weights, biases and z are in LDS
    for (int t0 = t_begin; t0 < t_end; t0 += TOK) {
      const bool valid = t0 + tf < a.NT;
      const int tok = lmap.token(min(t0 + tf, a.NT - 1));
      // weights, biases and the fragments of M are the same in every tile: reading them through an offset the
      // compiler cannot see through keeps the reads in the loop (hoisted, they would fill the register file)
      const int z0 = opaque_zero();
      const lds_frag_ptr w1t = w1f + z0, w2t = w2f + z0;
      const float *b1t = b1 + z0, *b2t = b2 + z0, *zt = zl + z0;
      __builtin_assume(b1t != nullptr);
      __builtin_assume(b2t != nullptr);
      float rs_ = 1.f, wp_ = 1.f;
      if constexpr (QUERY) {
        rs_ = a.rs[(int64_t)bh * a.N + tok];
        wp_ = a.wp[(int64_t)bh * a.N + tok];
      }
      const float wz_ = QUERY ? wp_ * rs_ : 1.f;             // dden_i = -(g_i . y_hat_i) / den_i

      // the map, recomputed: h (hi + lo), t = positive output before the slice powers; the ReLU gate is kept as one
      // bit per hidden unit, h itself goes to the B side tile right away
      f32x16 tt[T];
      unsigned gate[(T + 1) / 2];
      bf16x8 hpark[T][2];                               // h, kept until the tiles are free to take it
      {
        // between the two layers: barrier A1 (the second contraction of the tile before is done by then) and the
        // request for this tile's u rows (they are needed behind the map, and would not fit beside layer 1)
        u32x4 h_hi[T][2], h_lo[T][2];
        auto mid = [&]() {
          __syncthreads();
          request_u(t0);
        };
        mlp128_pipelined<ACT0, true>(xf, w1t, w2t, b1t, b2t, lane, g, a.act, h_hi, h_lo, tt, mid);
#pragma unroll
        for (int i = 0; i < (T + 1) / 2; ++i) gate[i] = 0u;
#pragma unroll
        for (int hb = 0; hb < T; ++hb)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            // h >= 0 after the ReLU: positive unless its bf16 pattern is a zero of either sign
            const unsigned half = (h_hi[hb][x >> 3][(x & 7) >> 1] >> (16 * (x & 1))) & 0x7fffu;
            gate[hb >> 1] |= (half != 0u ? 1u : 0u) << (16 * (hb & 1) + x);
          }
#pragma unroll
        for (int hb = 0; hb < T; ++hb) {
          hpark[hb][0] = __builtin_bit_cast(bf16x8, h_hi[hb][0]);
          hpark[hb][1] = __builtin_bit_cast(bf16x8, h_hi[hb][1]);
        }
      }
      __syncthreads();                                  // M1: the fragments of M have landed in the two tiles
      // dphi = rs (M u) + wz zvec   (the fragments of M come from L2: the next half block (lo or hi part of one
      // channel block, 8 fragments) is requested before the chain of the current one starts)
      f32x16 dv[T];
      {
        // steps of four fragments: step = 4 fb + 2 (0: lo part, 1: hi part) + (which half of the d contraction)
        constexpr int QF = KS / 2;
        bf16x8 mf[2][QF];
        auto request_m = [&](int step, bf16x8 (&dst)[QF]) {
          const int fb = step >> 2, hi = (step >> 1) & 1, q4 = step & 1;
#pragma unroll
          for (int i = 0; i < QF; ++i)
            dst[i] = hi ? frag_at(mhi, fb * KS + q4 * QF + i, lane) : frag_at(mlo, fb * KS + q4 * QF + i, lane);
        };
        request_m(0, mf[0]);
#pragma unroll
        for (int fb = 0; fb < T; ++fb) {
          f32x16 acc;
#pragma unroll
          for (int x = 0; x < 16; ++x) acc[x] = 0.f;
#pragma unroll
          for (int sub = 0; sub < 4; ++sub) {
            const int step = 4 * fb + sub;
            if (step + 1 < 4 * T) request_m(step + 1, mf[(step + 1) & 1]);
#pragma unroll
            for (int i = 0; i < QF; ++i) acc = mfma32(mf[step & 1][i], uf[(sub & 1) * QF + i], acc);
          }
#pragma unroll
          for (int x = 0; x < 16; ++x) dv[fb][x] = rs_ * acc[x] + wz_ * zt[32 * fb + crow(x, g)];
        }
      }
      // back through the slice powers and the activation: dv becomes du.  The slice power of a channel is wave-uniform
      // (it depends on the group of four registers only); the degrees the paper uses are compiled in, so that the
      // factor p t^(p-1) costs p - 1 multiplications and no selects.
      {
        float dots[4] = {0.f, 0.f, 0.f, 0.f};              // four chains instead of one of 64 dependent additions
        auto powers_back = [&](auto pc) {
          constexpr int PC = decltype(pc)::value;              // 0: any degree, taken at run time
          // (the degree of the general form goes through a value the compiler cannot see through, so that its
          // per-group exponents are formed inside this branch and not ahead of the dispatch for every degree)
          const int p_any = PC == 0 ? a.P + opaque_zero() : PC;
#pragma unroll
          for (int fb = 0; fb < T; ++fb)
#pragma unroll
            for (int x = 0; x < 16; ++x) {
              const float t0v = tt[fb][x];
              if constexpr (PC == 0) {
                const int extra = ((32 * fb + 8 * (x >> 2)) * p_any) / D;  // channel / Dp: slice power p = extra + 1
                dv[fb][x] *= (float)(extra + 1) * pow_small(t0v, extra);   // d/dt of t^p
              } else {
                constexpr int dummy = 0;
                (void)dummy;
                const int extra = ((32 * fb + 8 * (x >> 2)) * PC) / D;     // folds to a constant after unrolling
                float f = (float)(extra + 1);
                for (int i = 0; i < extra; ++i) f *= t0v;
                if (extra > 0) dv[fb][x] *= f;
              }
              dots[x & 3] += t0v * dv[fb][x];
            }
        };
        if (a.P == 1) powers_back(std::integral_constant<int, 1>{});
        else if (a.P == 2) powers_back(std::integral_constant<int, 2>{});
        else if (a.P == 4) powers_back(std::integral_constant<int, 4>{});
        else powers_back(std::integral_constant<int, 0>{});
        float dot = (dots[0] + dots[1]) + (dots[2] + dots[3]);
        if constexpr (ACT0) {
          dot = xhalf_sum(dot);
#pragma unroll
          for (int fb = 0; fb < T; ++fb)
#pragma unroll
            for (int x = 0; x < 16; ++x) dv[fb][x] = tt[fb][x] * (dv[fb][x] - dot);
        } else if (a.act == 1) {
#pragma unroll
          for (int fb = 0; fb < T; ++fb)
#pragma unroll
            for (int x = 0; x < 16; ++x) dv[fb][x] *= tt[fb][x];
        } else {
#pragma unroll
          for (int fb = 0; fb < T; ++fb)
#pragma unroll
            for (int x = 0; x < 16; ++x) dv[fb][x] = tt[fb][x] > 0.f ? dv[fb][x] : 0.f;
        }
      }
      bf16x8 dub[T][2];
      {
        const float keep = valid ? 1.f : 0.f;             // rows past the end of the token set contribute nothing
#pragma unroll
        for (int fb = 0; fb < T; ++fb)
#pragma unroll
          for (int sp = 0; sp < 2; ++sp) {
            u32x4 t4;
#pragma unroll
            for (int j = 0; j < 4; ++j) t4[j] = pack_bf16(dv[fb][8 * sp + 2 * j] * keep, dv[fb][8 * sp + 2 * j + 1] * keep);
            dub[fb][sp] = __builtin_bit_cast(bf16x8, t4);
          }
      }
      __syncthreads();                                  // M2: every wave has read its fragments of M
      write_chained(b_t, hpark);
      write_chained(a_t, dub);
      __syncthreads();                                  // B1: h and du are in place
      // dpre = (W2^T du) [h > 0], under the first contraction; the x rows come back from L2 meanwhile
      bf16x8 dpb[T][2];
      bf16x8 xp[KS];
      {
        // Software pipeline over the four hidden blocks: the fragments of block hb + 1 are requested (LDS; the last
        // two of the 32 from L2) before the matrix instructions of block hb, whose chain runs over the gating and
        // rounding of block hb - 1 (two accumulators take turns).
        bf16x8 wlast[T * T * 2 - W2T_LDS];
#pragma unroll
        for (int i = 0; i < T * T * 2 - W2T_LDS; ++i) wlast[i] = frag_at(w2tf, W2T_LDS + i, lane, z0);
        // this tile's x rows once more (L2): they go to the B side tile.  Requested behind the two fragments above:
        // loads return in order, and the last hidden block must not wait for these rows as well
        request_x(t0, xp);
        bf16x8 wt[2][2 * T];
        auto request_w = [&](int hb, bf16x8 (&dst)[2 * T]) {
#pragma unroll
          for (int i = 0; i < 2 * T; ++i) {
            const int idx = hb * T * 2 + i;
            if (idx < W2T_LDS) dst[i] = frag_at(w2tl, idx, lane);
            else dst[i] = wlast[idx - W2T_LDS];
          }
        };
        // the ReLU gate (bit -> sign position -> select) and the rounding in pairs of one finished block
        auto finish = [&](int hb, const f32x16 &acc) {
          const unsigned gbits = gate[hb >> 1] >> (16 * (hb & 1));
          auto gated = [&](int x) { return (int)(gbits << (31 - x)) < 0 ? acc[x] : 0.f; };
#pragma unroll
          for (int sp = 0; sp < 2; ++sp) {
            u32x4 t4;
#pragma unroll
            for (int j = 0; j < 4; ++j) t4[j] = pack_bf16(gated(8 * sp + 2 * j), gated(8 * sp + 2 * j + 1));
            dpb[hb][sp] = __builtin_bit_cast(bf16x8, t4);
          }
        };
        f32x16 accs[2];
        request_w(0, wt[0]);
#pragma unroll
        for (int hb = 0; hb < T; ++hb) {
          f32x16 &acc = accs[hb & 1];
#pragma unroll
          for (int x = 0; x < 16; ++x) acc[x] = 0.f;
          if (hb + 1 < T) request_w(hb + 1, wt[(hb + 1) & 1]);
          if (hb == 1) request_x(t0 + TOK, xf);         // the rows of the next tile
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int fb = 0; fb < T; ++fb)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
              acc = mfma32(wt[hb & 1][fb * 2 + s2], dub[fb][s2], acc);
              // a quarter of the previous block's finish behind every second matrix instruction
              if (hb > 0 && s2 == 1) {
                const f32x16 &prev = accs[(hb - 1) & 1];
                const unsigned gbits = gate[(hb - 1) >> 1] >> (16 * ((hb - 1) & 1));
                auto gated = [&](int x) { return (int)(gbits << (31 - x)) < 0 ? prev[x] : 0.f; };
                const int sp = fb >> 1, j0 = 2 * (fb & 1);
                u32x4 t4 = {0u, 0u, 0u, 0u};
                if (j0 != 0) t4 = __builtin_bit_cast(u32x4, dpb[hb - 1][sp]);   // (the first half was set a step earlier)
                t4[j0] = pack_bf16(gated(8 * sp + 2 * j0), gated(8 * sp + 2 * j0 + 1));
                t4[j0 + 1] = pack_bf16(gated(8 * sp + 2 * j0 + 2), gated(8 * sp + 2 * j0 + 3));
                dpb[hb - 1][sp] = __builtin_bit_cast(bf16x8, t4);
              }
            }
          __builtin_amdgcn_sched_barrier(0);
        }
        finish(T - 1, accs[(T - 1) & 1]);
      }
      __syncthreads();                                  // A2: the first contraction has read both tiles
      write_chained(a_t, dpb);
      {
        const int sw_now = row_sw + opaque_zero();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)                 // x: channels 16 ks + 8 g .. + 7 = piece 2 ks + g of the row
          *reinterpret_cast<bf16x8 *>(b_t + row_off + (((2 * ks + g) ^ sw_now) << 4)) = xp[ks];
      }
      __syncthreads();                                  // B2: dpre and x are in place
    }
    return;
  }

  // =============================== the two contractions over the tokens (waves 4 .. 7) ===============================
  f32x16 acc2[NCB], acc1[NCB];
#pragma unroll
  for (int i = 0; i < NCB; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      acc2[i][x] = 0.f;
      acc1[i][x] = 0.f;
    }
  // transposing reads: lane = (group m, i, a), see ds_read_tr.  A fragment half covers rows T0 + i, T0 = 16 ks + 8 g
  // + 4 jj, so psw(T0 + i) = 4 i + (2 g + jj) % 4 is a per-lane constant per half; k-steps are immediates
  const int tm = lane >> 4, ti = (lane >> 2) & 3, ta = lane & 3, tg = tm >> 1;
  auto tr_base = [&](int blk, int jj) {
    return (8 * tg + ti) * ROWB + (((4 * blk + 2 * (tm & 1) + (ta >> 1)) ^ (4 * ti + ((2 * tg + jj) & 3))) << 4) + 8 * (ta & 1);
  };
  int ab[2], bb[T][2];
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    ab[jj] = tr_base(w, jj);
#pragma unroll
    for (int cb = 0; cb < T; ++cb) bb[cb][jj] = tr_base(cb, jj);
  }
  const __bf16 one = static_cast<__bf16>(r == 0 ? 1.0f : 0.0f);     // the "1" column that yields the bias gradient
  const bf16x8 ones = bf16x8{one, one, one, one, one, one, one, one};
  // row block w of (A side)^T (B side | 1): one 16-token slice (5 matrix instructions) per batch, the 10 transposing
  // reads of the next batch placed behind the matrix instructions of the current one
  auto contract = [&](f32x16 (&acc)[NCB]) {
    constexpr int NBATCH = TOK / 16;
    bf16x8 fr[2][NCB];                               // [buffer][operand]: operand 0 = A side, 1 + cb = B side
    auto rd = [&](int batch, int buf, int op) {
      const int off = batch * 16 * ROWB;
      fr[buf][op] = op == 0 ? join(ds_read_tr(a_t, ab[0] + off), ds_read_tr(a_t, ab[1] + off + 4 * ROWB))
                            : join(ds_read_tr(b_t, bb[op - 1][0] + off), ds_read_tr(b_t, bb[op - 1][1] + off + 4 * ROWB));
    };
#pragma unroll
    for (int i = 0; i < NCB; ++i) rd(0, 0, i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int batch = 0; batch < NBATCH; ++batch) {
      const int buf = batch & 1;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        acc[cb] = mfma32(fr[buf][0], cb < T ? fr[buf][1 + cb] : ones, acc[cb]);
        if (batch + 1 < NBATCH) rd(batch + 1, buf ^ 1, cb);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  __syncthreads();                                    // weights, biases and z are in LDS
  for (int t0 = t_begin; t0 < t_end; t0 += TOK) {
    __syncthreads();                                  // A1
    // M (natural-order fragments, hi and lo part, 32 KiB each) into the two tiles, which are free until h and du arrive
    dma_to_lds(a.m_hi + (int64_t)bh * (D * D / 8), reinterpret_cast<bf16x8 *>(a_t), D * D / 8 / 64, w, 4, lane);
    dma_to_lds(a.m_lo + (int64_t)bh * (D * D / 8), reinterpret_cast<bf16x8 *>(b_t), D * D / 8 / 64, w, 4, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                  // M1
    __syncthreads();                                  // M2
    __syncthreads();                                  // B1
    contract(acc2);
    __syncthreads();                                  // A2
    __syncthreads();                                  // B2
    contract(acc1);
  }
  {
    float *dst = a.part + (((int64_t)bh * gridDim.x + chunk) * NSET) * NT2 * 1024 + (int64_t)w * NCB * 1024;
#pragma unroll
    for (int i = 0; i < NCB; ++i)
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        dst[i * 1024 + x * 64 + lane] = acc2[i][x];
        dst[(NT2 + i) * 1024 + x * 64 + lane] = acc1[i][x];
      }
  }
}

// ------------------------------------------------------------------------------------------------
// grad_reduce_kernel: grid (T*(T+1)*1024 / 256, n_out).  Output o sums set `set` of the partials over the
// chunks of (batch b, head o) for every b (n_sum = B, shared parameters) or of (batch, head) pair o alone
// (n_sum = 1), in a fixed order.  mat[o][row][col] row-major fp32, vec[o][row] = the extra column block
// (columns 0 and 1: the hi and lo parts of a weighted sum, or the plain sum and zero).
// With mat1 given the launch has a third grid dimension: z = 1 sums set `set + 1` into (mat1, vec1).
__global__ __launch_bounds__(256) void grad_reduce_kernel(const float *__restrict__ part, float *__restrict__ mat,
                                                          float *__restrict__ vec, int D, int n_chunks, int n_sets,
                                                          int set, int n_sum, int stride_sum, float *__restrict__ mat1 = nullptr,
                                                          float *__restrict__ vec1 = nullptr, __bf16 *__restrict__ frag_hi = nullptr,
                                                          __bf16 *__restrict__ frag_lo = nullptr) {
  if (blockIdx.z == 1) {
    mat = mat1;
    vec = vec1;
    set += 1;
  }
  const int T = D / 32, NCB = T + 1, NT2 = T * NCB;
  const int o = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= NT2 * 1024) return;
  const int ti = e >> 10, x = (e >> 6) & 15, lane = e & 63, r = lane & 31, g = lane >> 5;
  const int rb = ti / NCB, cb = ti % NCB;
  if (cb == T && r != 0) return;
  // four chunks per step: the loads of a step do not depend on each other (a plain running sum exposes one
  // memory round trip per chunk); the order of the additions is fixed all the same
  float sum = 0.f;
  const int64_t cstride = (int64_t)n_sets * NT2 * 1024;
  const bool two = cb == T;
  for (int b = 0; b < n_sum; ++b) {
    const int64_t bh = (int64_t)b * stride_sum + o;
    const float *src = part + ((bh * n_chunks) * n_sets + set) * (int64_t)NT2 * 1024 + e;
    int c = 0;
    for (; c + 4 <= n_chunks; c += 4) {
      float v[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = src[(c + i) * cstride];
        u[i] = two ? src[(c + i) * cstride + 1] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) sum += v[i] + u[i];
    }
    for (; c < n_chunks; ++c) sum += src[c * cstride] + (two ? src[c * cstride + 1] : 0.f);
  }
  const int row = 32 * rb + crow(x, g);
  if (cb < T) {
    const int col = 32 * cb + r;
    mat[((int64_t)o * D + row) * D + col] = sum;
    if (frag_hi) {
      // the same matrix as hi + lo natural-order fragments (see natural_frags_kernel), for the pass that reads it next
      const int lane_f = ((col >> 3) & 1) * 32 + (row & 31);
      const int64_t fi = (int64_t)o * D * D + ((((row >> 5) * (D / 16) + (col >> 4)) * 64 + lane_f) << 3) + (col & 7);
      const __bf16 hpart = static_cast<__bf16>(sum);
      frag_hi[fi] = hpart;
      frag_lo[fi] = static_cast<__bf16>(sum - static_cast<float>(hpart));
    }
  } else {
    vec[(int64_t)o * D + row] = sum;
  }
}

// ------------------------------------------------------------------------------------------------
// host side

template <typename T>
static inline T *ws_ptr(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }
static inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

void make_grad_plan(const Plan &pl, size_t base_off, GradPlan &gp) {
  const size_t BH = (size_t)pl.B * pl.H;
  const int D = pl.D, T = D / 32;
  gp.tiles_per_set = T * (T + 1);
  auto chunking = [&](int n_tok, int &CH, int &n_chunks) {
    const int tiles = (n_tok + 127) / 128;
    const int per_head = 256 / (int)BH > 0 ? 256 / (int)BH : 1;
    const int want = tiles < per_head ? (tiles > 0 ? tiles : 1) : per_head;
    CH = ((tiles + want - 1) / want) * 128;
    if (CH < 128) CH = 128;
    n_chunks = (n_tok + CH - 1) / CH;
  };
  chunking(pl.N, gp.CHq, gp.n_chunks_q);
  chunking(pl.NL, gp.CHk, gp.n_chunks_k);
  size_t off = base_off;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  gp.off_w2tq = take((size_t)pl.H * D * D * 2);
  gp.off_w2tk = take((size_t)pl.H * D * D * 2);
  gp.off_shi = take(BH * D * D * 2);
  gp.off_slo = take(BH * D * D * 2);
  gp.off_dS = take(BH * D * D * 4);
  gp.off_dz = take(BH * D * 4);
  gp.off_dshi = take(BH * D * D * 2);
  gp.off_dslo = take(BH * D * D * 2);
  gp.off_gsign = take(BH * pl.N * D * 2);
  gp.off_rs = take(BH * pl.N * 4);
  gp.off_wp = take(BH * pl.N * 4);
  const size_t pq = BH * gp.n_chunks_q * 2 * gp.tiles_per_set * 1024 * 4;
  const size_t pk = BH * gp.n_chunks_k * 2 * gp.tiles_per_set * 1024 * 4;
  gp.off_part = take(pq > pk ? pq : pk);
  gp.total = off;
}

hipError_t launch_fill_zero(float *p, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  fill_zero_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, (int64_t)n);
  return hipGetLastError();
}

hipError_t launch_vd_rows(const Plan &pl, const void *y_teacher, const void *y_student, const float *row_den, void *gsign,
                          float *rs, float *wp, hipStream_t st, double *l1_partial, double *loss) {
  if (l1_partial && !pl.f32) {
    dim3 grid(kL1Parts, pl.B * pl.H);
    if (pl.D == 64)
      vd_rows_loss_kernel<64><<<grid, 256, 0, st>>>(y_teacher, y_student, row_den, static_cast<bf16x8 *>(gsign), rs, wp, l1_partial,
                                                    pl.H, pl.N, pl.sb, pl.sh, pl.sn);
    else
      vd_rows_loss_kernel<128><<<grid, 256, 0, st>>>(y_teacher, y_student, row_den, static_cast<bf16x8 *>(gsign), rs, wp, l1_partial,
                                                     pl.H, pl.N, pl.sb, pl.sh, pl.sn);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_l1_final(pl, l1_partial, loss, st);
  }
  const int D = pl.D, rpb = 256 / (D / 8);
  dim3 grid((pl.N + rpb - 1) / rpb, pl.B * pl.H);
#define HA_ROWS(DD, F32) \
  vd_rows_kernel<DD, F32><<<grid, 256, 0, st>>>(y_teacher, y_student, row_den, static_cast<bf16x8 *>(gsign), rs, wp, pl.H, pl.N, \
                                                pl.sb, pl.sh, pl.sn)
  if (D == 64) { if (pl.f32) HA_ROWS(64, true); else HA_ROWS(64, false); }
  else { if (pl.f32) HA_ROWS(128, true); else HA_ROWS(128, false); }
#undef HA_ROWS
  return hipGetLastError();
}

hipError_t launch_natural_frags(const float *M, void *hi, void *lo, int rows, int cols, int n_mat, hipStream_t st) {
  dim3 grid((rows * cols + 255) / 256, n_mat);
  natural_frags_kernel<<<grid, 256, 0, st>>>(M, static_cast<__bf16 *>(hi), static_cast<__bf16 *>(lo), rows, cols);
  return hipGetLastError();
}

// Everything after the student's forward: S, z are in the forward's workspace region (`pl` offsets), y_teacher,
// y_student and row_den hold the two outputs and the student's row denominators.
hipError_t launch_value_distill_backward(const Plan &pl, const GradPlan &gp, const void *q, const void *k, const void *v,
                                         const ha_feature_map &phi_q, const ha_feature_map &phi_k, const void *y_teacher,
                                         const void *y_student, const float *row_den, const ha_feature_map_grad &gq,
                                         const ha_feature_map_grad &gk, void *ws, hipStream_t st, double *l1_partial,
                                         double *loss) {
  const int D = pl.D, BH = pl.B * pl.H;
  hipError_t e;
#define HA_CHECK() if ((e = hipGetLastError()) != hipSuccess) return e
  // operand fragments: W1, W2 of both maps (forward order), W2^T (chained), S (natural, hi + lo): one launch
  {
    GradOperands o;
    o.w1q = phi_q.w1; o.w2q = phi_q.w2; o.w1k = phi_k.w1; o.w2k = phi_k.w2;
    o.w1qf = ws_ptr<__bf16>(ws, pl.off_w1q); o.w2qf = ws_ptr<__bf16>(ws, pl.off_w2q);
    o.w1kf = ws_ptr<__bf16>(ws, pl.off_w1k); o.w2kf = ws_ptr<__bf16>(ws, pl.off_w2k);
    o.w2tq = ws_ptr<__bf16>(ws, gp.off_w2tq); o.w2tk = ws_ptr<__bf16>(ws, gp.off_w2tk);
    o.S = ws_ptr<float>(ws, pl.off_S); o.s_hi = ws_ptr<__bf16>(ws, gp.off_shi); o.s_lo = ws_ptr<__bf16>(ws, gp.off_slo);
    o.D = D; o.H = pl.H;
    dim3 grid((D * D + 255) / 256, 4 * pl.H + BH);
    if (pl.f32) grad_operands_kernel<true><<<grid, 256, 0, st>>>(o);
    else grad_operands_kernel<false><<<grid, 256, 0, st>>>(o);
    HA_CHECK();
  }
  // per-row factors
  if ((e = launch_vd_rows(pl, y_teacher, y_student, row_den, ws_ptr<void>(ws, gp.off_gsign), ws_ptr<float>(ws, gp.off_rs),
                          ws_ptr<float>(ws, gp.off_wp), st, l1_partial, loss)) != hipSuccess)
    return e;
  GradArgs a;
  a.H = pl.H; a.N = pl.N; a.R = pl.R; a.G = pl.G; a.P = pl.P;
  a.sb = pl.sb; a.sh = pl.sh; a.sn = pl.sn;
  a.part = ws_ptr<float>(ws, gp.off_part);
  a.rs = ws_ptr<float>(ws, gp.off_rs);
  a.wp = ws_ptr<float>(ws, gp.off_wp);
  const dim3 rgrid2(gp.tiles_per_set * 1024 / 256, pl.H, 2), rgrid_bh(gp.tiles_per_set * 1024 / 256, BH);
  // query pass: phi_q's gradient and [dS | dz]
  {
    a.x = q; a.u = ws_ptr<void>(ws, gp.off_gsign);
    a.w1f = ws_ptr<bf16x8>(ws, pl.off_w1q); a.w2f = ws_ptr<bf16x8>(ws, pl.off_w2q); a.w2tf = ws_ptr<bf16x8>(ws, gp.off_w2tq);
    a.b1 = phi_q.b1; a.b2 = phi_q.b2;
    a.m_hi = ws_ptr<bf16x8>(ws, gp.off_shi); a.m_lo = ws_ptr<bf16x8>(ws, gp.off_slo);
    a.zvec = ws_ptr<float>(ws, pl.off_z);
    a.NT = pl.N; a.CH = gp.CHq; a.act = pl.act_q;
    dim3 grid(gp.n_chunks_q, BH);
    if (D == 64) { if (pl.f32) grad_kernel<64, true, true><<<grid, 256, 0, st>>>(a); else grad_kernel<64, false, true><<<grid, 256, 0, st>>>(a); }
    else if (a.act == HA_ACT_SOFTMAX) { if (pl.f32) grad_split_kernel<true, true, true><<<grid, 512, 0, st>>>(a); else grad_split_kernel<false, true, true><<<grid, 512, 0, st>>>(a); }
    else { if (pl.f32) grad_split_kernel<true, true, false><<<grid, 512, 0, st>>>(a); else grad_split_kernel<false, true, false><<<grid, 512, 0, st>>>(a); }
    HA_CHECK();
    grad_reduce_kernel<<<rgrid2, 256, 0, st>>>(a.part, gq.w2, gq.b2, D, gp.n_chunks_q, 2, 0, pl.B, pl.H, gq.w1, gq.b1);
    HA_CHECK();
    // [dS | dz]: the weighted state pass over all query tokens, reduced per (batch, head)
    if ((e = launch_weighted_state(pl, q, ws_ptr<void>(ws, gp.off_gsign), a.rs, a.wp, phi_q, a.w1f, a.w2f, a.part, gp.CHq,
                                   gp.n_chunks_q, st)) != hipSuccess)
      return e;
    grad_reduce_kernel<<<rgrid_bh, 256, 0, st>>>(a.part, ws_ptr<float>(ws, gp.off_dS), ws_ptr<float>(ws, gp.off_dz), D,
                                                 gp.n_chunks_q, 1, 0, 1, 0, nullptr, nullptr, ws_ptr<__bf16>(ws, gp.off_dshi),
                                                 ws_ptr<__bf16>(ws, gp.off_dslo));
    HA_CHECK();
  }
  // key pass over the linear tokens: phi_k's gradient
  {
    a.x = k; a.u = v;
    a.w1f = ws_ptr<bf16x8>(ws, pl.off_w1k); a.w2f = ws_ptr<bf16x8>(ws, pl.off_w2k); a.w2tf = ws_ptr<bf16x8>(ws, gp.off_w2tk);
    a.b1 = phi_k.b1; a.b2 = phi_k.b2;
    a.m_hi = ws_ptr<bf16x8>(ws, gp.off_dshi); a.m_lo = ws_ptr<bf16x8>(ws, gp.off_dslo);
    a.zvec = ws_ptr<float>(ws, gp.off_dz);
    a.NT = pl.NL; a.CH = gp.CHk; a.act = pl.act_k;
    dim3 grid(gp.n_chunks_k, BH);
    if (D == 64) { if (pl.f32) grad_kernel<64, true, false><<<grid, 256, 0, st>>>(a); else grad_kernel<64, false, false><<<grid, 256, 0, st>>>(a); }
    else if (a.act == HA_ACT_SOFTMAX) { if (pl.f32) grad_split_kernel<true, false, true><<<grid, 512, 0, st>>>(a); else grad_split_kernel<false, false, true><<<grid, 512, 0, st>>>(a); }
    else { if (pl.f32) grad_split_kernel<true, false, false><<<grid, 512, 0, st>>>(a); else grad_split_kernel<false, false, false><<<grid, 512, 0, st>>>(a); }
    HA_CHECK();
    grad_reduce_kernel<<<rgrid2, 256, 0, st>>>(a.part, gk.w2, gk.b2, D, gp.n_chunks_k, 2, 0, pl.B, pl.H, gk.w1, gk.b1);
    HA_CHECK();
  }
#undef HA_CHECK
  return hipSuccess;
}

}  // namespace ha
