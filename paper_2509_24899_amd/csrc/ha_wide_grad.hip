// Gradient of the value-distillation loss (Attention Surgery, Sec. 3.3: Eq. "vd_loss", update line of Alg. "distil")
// for two-layer feature maps of any width the layer-by-layer forward handles (Tab. "phi": the default 256-wide map,
// P = 3, 4, ...), gfx950.  Same mathematics as ha_grad.hip; here every step is a pass of its own over register
// images in HBM (layout: ha_wide.hip), per side (queries, then linear keys) right after that side's forward passes
// have been re-run so that its hidden activations h, pre-activations u and phi are in the workspace:
//
//   wide_dphi_kernel        dphi = rs (M u) + wz zvec per 256-channel block, t = activation(u), phi_q = t^p for the dS
//                           product, and du = t dt - t (sum over all channels of t dt) as a bf16 image; only a softmax
//                           over more than 256 channels needs the sum from other workgroups: then t replaces u in place,
//                           t dt goes to a second fp32 image, its per-token sum over the block aside, and
//   wide_du_kernel          finishes du = t dt - t (sum over all blocks) -> bf16
//   wide_back_layer_kernel  dpre = (W2^T du) [h > 0] -> bf16        (W2^T fragments staged through LDS)
//   wide_contract_kernel    sum over tokens of  A^T [B | 1]  for  (du, h) -> dW2, db2;  (dpre, x) -> dW1, db1;
//                           queries also (rs phi_q, [g | wp]) -> dS, dz.  A from an image, B from an image or from
//                           rows; one 128 x 128 slab of the product per workgroup, partial tiles per chunk of tokens
//   wide_grad_reduce_kernel fixed-order sum of the partial tiles over chunks (and the batch) -> row-major fp32
#include "ha_device.h"
#include "ha_plan.h"

namespace ha {

// ------------------------------------------------------------------------------------------------
// wide_prep_t_kernel: grid (ceil(F*K / 256), H).  W [H][F][K] (io dtype) -> fragments of W^T [K x F] in chained order:
//   wt[h][ob][fb][s][lane][t] = W[h][32 fb + crow(8 s + t, g)][32 ob + r]
template <bool F32>
__global__ __launch_bounds__(256) void wide_prep_t_kernel(const void *__restrict__ wsrc, __bf16 *__restrict__ wt, int F, int K) {
  const int h = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= F * K) return;
  const int t = e & 7, lane = (e >> 3) & 63, rest = e >> 9;
  const int r = lane & 31, g = lane >> 5;
  const int FB = F / 32;
  const int s = rest & 1, fb = (rest >> 1) % FB, ob = (rest >> 1) / FB;
  const int64_t src = ((int64_t)h * F + 32 * fb + crow(8 * s + t, g)) * K + 32 * ob + r;
  float val;
  if constexpr (F32) val = static_cast<const float *>(wsrc)[src];
  else val = static_cast<float>(static_cast<const __bf16 *>(wsrc)[src]);
  wt[(int64_t)h * F * K + e] = static_cast<__bf16>(val);
}

struct WideGradArgs {
  const void *x;                  // q or k rows (io dtype, strided)
  const void *u;                  // queries: sign tensor, bf16 dense [B*H][N][D]; keys: v rows (io dtype, strided)
  const float *rs, *wp;           // queries: [B*H][N]
  const bf16x8 *m_hi, *m_lo;      // [B*H][F*D/8]: natural-order fragments of S (queries) or dS (keys)
  const float *zvec;              // [B*H][F]
  f32x4 *t_img;                   // in: pre-activations u; out: t = activation(u)            [bh][tb][F/32][4][64]
  f32x4 *tdt_img;                 // out: t dt (softmax), dt t (exp), dt [u > 0] (relu)
  const float *stat;              // softmax maxima / sums per 256-channel block (last layer of the forward)
  float *pdot;                    // [bh][tb][blocks][64]: per-token sum of t dt over the block's channels
  bf16x8 *du_img;                 // FUSED: du, bf16 image
  bf16x8 *phi_img;                // QUERY: phi_q, bf16 image (zero for tokens past the end)
  int H, N, F, n_tok, n_tb, R, G, P, act;
  int64_t sb, sh, sn;
};

// ------------------------------------------------------------------------------------------------
// wide_dphi_kernel: grid (ceil(n_tb / 4), ceil(F / 256), B*H), one 32-token block per wave.
// FUSED (every case but a softmax over more than one 256-channel block): the sum of the softmax Jacobian is complete
// inside the workgroup's block, so du is formed here (t dt of the eight tiles waits in registers for the sum, t is
// recomputed from the pre-activations, which the wave has just read) and written as the bf16 image; the fp32 side
// images and wide_du_kernel are not needed.  QUERY: phi_q = t^p is written as a bf16 image for the dS product.
template <int D, bool F32, bool QUERY, bool FUSED>
__global__ __launch_bounds__(256) void wide_dphi_kernel(WideGradArgs a) {
  constexpr int KS = D / 16, NT = 8;
  const int bh = blockIdx.z, h = bh % a.H;
  const int lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
  const int tb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tb >= a.n_tb) return;
  const int FB = a.F / 32, nblk = (a.F + 255) / 256;
  const int fb0 = blockIdx.y * NT, nt = min(NT, FB - fb0);
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const LinearMap lmap(QUERY ? 0 : a.R, a.G);
  const bool valid = 32 * tb + r < a.n_tok;
  const int tok = lmap.token(min(32 * tb + r, a.n_tok - 1));
  bf16x8 uf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    if constexpr (QUERY) uf[ks] = static_cast<const bf16x8 *>(a.u)[((int64_t)bh * a.N + tok) * (D / 8) + 2 * ks + g];
    else uf[ks] = load8<F32>(a.u, base + (int64_t)tok * a.sn + 16 * ks + 8 * g);
  }
  float rs_ = 1.f, wz_ = 1.f;
  if constexpr (QUERY) {
    rs_ = a.rs[(int64_t)bh * a.N + tok];
    wz_ = a.wp[(int64_t)bh * a.N + tok] * rs_;
  }
  float off = 0.f, inv = 1.f;
  if (a.act == 0) {
    const float *st = a.stat + (((int64_t)bh * a.n_tb + tb) * nblk * 2) * 64 + lane;
    float m = -INFINITY;
    for (int b = 0; b < nblk; ++b) m = fmaxf(m, st[b * 128]);
    float sum = 0.f;
    for (int b = 0; b < nblk; ++b) sum += st[b * 128 + 64] * fast_exp2((st[b * 128] - m) * kLog2e);
    off = -m * kLog2e;
    inv = 1.0f / sum;
  }
  const GlobalFrags mhi = global_frags(a.m_hi + (int64_t)bh * ((int64_t)a.F * D / 8), a.F * D * 2);
  const GlobalFrags mlo = global_frags(a.m_lo + (int64_t)bh * ((int64_t)a.F * D / 8), a.F * D * 2);
  const float inv_groups = 8.0f * (float)a.P / (float)a.F;
  auto activation = [&](float u) {
    if (a.act == 0) return fast_exp2(__builtin_fmaf(u, kLog2e, off)) * inv;
    if (a.act == 1) return fast_exp2(u * kLog2e);
    return fmaxf(u, 0.f);
  };
  float pdot = 0.f;
  f32x16 keep[FUSED ? NT : 1];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    if (j >= nt) break;
    const int fb = fb0 + j;
    f32x16 acc;
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[x] = 0.f;
    bf16x8 fl[KS], fh[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      fl[ks] = frag_at(mlo, fb * KS + ks, lane);
      fh[ks] = frag_at(mhi, fb * KS + ks, lane);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      acc = mfma32(fl[ks], uf[ks], acc);
      acc = mfma32(fh[ks], uf[ks], acc);
    }
    const int64_t img = (((int64_t)bh * a.n_tb + tb) * FB + fb) * 4;
    f32x16 phi;
#pragma unroll
    for (int x4 = 0; x4 < 4; ++x4) {
      const f32x4 uq = a.t_img[(img + x4) * 64 + lane];
      const int extra = (int)(((float)(4 * fb + x4) + 0.5f) * inv_groups);        // slice power - 1, wave-uniform
      f32x4 tq, dq;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = 32 * fb + crow(4 * x4 + i, g);
        const float dphi = rs_ * acc[4 * x4 + i] + wz_ * a.zvec[(int64_t)bh * a.F + c];
        const float t = activation(uq[i]);
        const float t2 = t * t;
        float pw = (extra & 1) ? t : 1.f;                                        // t^extra
        pw = (extra & 2) ? pw * t2 : pw;
        pw = (extra & 4) ? pw * (t2 * t2) : pw;
        const float dt = dphi * (float)(extra + 1) * pw;
        float v;
        if (a.act == 2) v = uq[i] > 0.f ? dt : 0.f;
        else v = t * dt;
        v = valid ? v : 0.f;
        tq[i] = t;
        dq[i] = v;
        phi[4 * x4 + i] = valid ? pw * t : 0.f;
        pdot += v;
      }
      if constexpr (FUSED) {
#pragma unroll
        for (int i = 0; i < 4; ++i) keep[j][4 * x4 + i] = dq[i];
      } else {
        a.t_img[(img + x4) * 64 + lane] = tq;
        a.tdt_img[(img + x4) * 64 + lane] = dq;
      }
    }
    if constexpr (QUERY) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        f32x8 o;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = phi[8 * s + i];
        a.phi_img[(img / 4 * 2 + s) * 64 + lane] = __builtin_convertvector(o, bf16x8);
      }
    }
  }
  pdot = xhalf_sum(pdot);
  if constexpr (!FUSED) {
    a.pdot[(((int64_t)bh * a.n_tb + tb) * nblk + blockIdx.y) * 64 + lane] = pdot;
  } else {
    const float dot = a.act == 0 ? pdot : 0.f;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if (j >= nt) break;
      const int64_t img = (((int64_t)bh * a.n_tb + tb) * FB + fb0 + j) * 4;
      if (a.act == 0) {
#pragma unroll
        for (int x4 = 0; x4 < 4; ++x4) {
          const f32x4 uq = a.t_img[(img + x4) * 64 + lane];
#pragma unroll
          for (int i = 0; i < 4; ++i) keep[j][4 * x4 + i] -= activation(uq[i]) * dot;
        }
      }
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        f32x8 o;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = keep[j][8 * s + i];
        a.du_img[(img / 4 * 2 + s) * 64 + lane] = __builtin_convertvector(o, bf16x8);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// wide_du_kernel: grid (ceil(n_tb / 4), B*H).  du = t dt - t sum(t dt) for the softmax, t dt as it is otherwise; bf16 image.
__global__ __launch_bounds__(256) void wide_du_kernel(const f32x4 *__restrict__ t_img, const f32x4 *__restrict__ tdt_img,
                                                      const float *__restrict__ pdot, bf16x8 *__restrict__ du, int F, int n_tb,
                                                      int act) {
  const int bh = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int tb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tb >= n_tb) return;
  const int FB = F / 32, nblk = (F + 255) / 256;
  float dot = 0.f;
  if (act == 0)
    for (int b = 0; b < nblk; ++b) dot += pdot[(((int64_t)bh * n_tb + tb) * nblk + b) * 64 + lane];
  for (int fb = 0; fb < FB; ++fb) {
    const int64_t img = (((int64_t)bh * n_tb + tb) * FB + fb) * 4;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      f32x8 o;
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const f32x4 tq = t_img[(img + 2 * s + x) * 64 + lane], dq = tdt_img[(img + 2 * s + x) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[4 * x + i] = dq[i] - tq[i] * dot;
      }
      du[(img / 4 * 2 + s) * 64 + lane] = __builtin_convertvector(o, bf16x8);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// wide_back_layer_kernel: grid (ceil(n_tb / 4), ceil(NOUT / 256), B*H), 4 waves.  dpre^T = (W^T du^T) gated by the
// hidden activations of the forward: input du as a bf16 image of width K, W^T [NOUT x K] fragments (chained
// order) staged through LDS as in wide_layer_kernel, h_hi image of width NOUT for the gate, output bf16 image.
__global__ __launch_bounds__(256, 2) void wide_back_layer_kernel(const bf16x8 *__restrict__ du, const bf16x8 *__restrict__ wt_all,
                                                                 const bf16x8 *__restrict__ h_hi, bf16x8 *__restrict__ dpre, int H,
                                                                 int K, int NOUT, int n_tb) {
  constexpr int NT = 8, KCH = 2, STG = NT * KCH * 2 * 64;
  __shared__ bf16x8 wl[2][STG];
  const int bh = blockIdx.z, h = bh % H;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool live = blockIdx.x * 4 + w < n_tb;
  const int tb = live ? blockIdx.x * 4 + w : n_tb - 1;
  const int KB = K / 32, OB = NOUT / 32;
  const int ob0 = blockIdx.y * NT;
  const int nt = min(NT, OB - ob0);
  const bf16x8 *wg = wt_all + (int64_t)h * ((int64_t)NOUT * K / 8);
  const bf16x8 *bsrc = du + ((int64_t)bh * n_tb + tb) * KB * 128 + lane;
  f32x16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  auto stage = [&](int c, int buf) {
    for (int j = 0; j < nt; ++j)
      dma_to_lds(wg + (((int64_t)(ob0 + j) * KB + c * KCH) * 2) * 64, &wl[buf][j * KCH * 2 * 64], KCH * 2, w, 4, lane);
  };
  bf16x8 cb[2], nb[2];
  stage(0, 0);
  cb[0] = bsrc[0];
  cb[1] = bsrc[64];
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  const int n_stages = KB / KCH;
  for (int c = 0; c < n_stages; ++c) {
    if (c + 1 < n_stages) stage(c + 1, (c + 1) & 1);
    const bf16x8 *wbuf = &wl[c & 1][lane];
#pragma unroll
    for (int kbl = 0; kbl < KCH; ++kbl) {
      const int kb = c * KCH + kbl;
      if (kb + 1 < KB) {
        nb[0] = bsrc[((kb + 1) * 2) * 64];
        nb[1] = bsrc[((kb + 1) * 2 + 1) * 64];
      }
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          if (j < nt) acc[j] = mfma32(wbuf[(j * KCH * 2 + kbl * 2 + s) * 64], cb[s], acc[j]);
      cb[0] = nb[0];
      cb[1] = nb[1];
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  if (!live) return;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    if (j >= nt) break;
    const int64_t blk = ((int64_t)bh * n_tb + tb) * OB + ob0 + j;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const bf16x8 hh = h_hi[(blk * 2 + s) * 64 + lane];
      f32x8 o;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = static_cast<float>(hh[i]) > 0.f ? acc[j][8 * s + i] : 0.f;
      dpre[(blk * 2 + s) * 64 + lane] = __builtin_convertvector(o, bf16x8);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// wide_contract_kernel: grid (n_chunks, B*H, (WA / 128) * (WB / 128)), 4 waves.  Per 128-token tile the A slab
// (128 rows of the A image, tokens as columns) and the B slab (128 columns) are parked in LDS with tokens contiguous,
// as in the state pass, and wave w contracts row block w of the slab with the four column blocks and the extra
// column block.  BSRC 0: B from a bf16 image of width WB; 1: rows of an io-dtype tensor behind the token map (q / k,
// width D); 2: rows of the dense bf16 sign tensor.  a_scale (optional, [B*H][N]): per-token factor on A before it is
// rounded (the 1 / den_i of the dS product).  Extra column block: ones, or with wcol the (hi, lo) pair of wcol's entry.
// Partial tiles: part[bh][chunk][slab pair][w][5][16][64].
struct ContractArgs {
  const bf16x8 *a_img;       // [bh][tb][WA/32][2][64]
  const float *a_scale;      // or null
  const bf16x8 *b_img;       // BSRC 0
  const void *b_rows;        // BSRC 1 (io dtype, strided) / 2 (bf16 dense [B*H][N][D])
  const float *wcol;         // or null
  float *part;
  int H, N, WA, WB, n_tok, n_tb, R, G, CH;
  int64_t sb, sh, sn;
};

template <int BSRC, bool F32>
__global__ __launch_bounds__(256, 1) void wide_contract_kernel(ContractArgs a) {
  constexpr int TOK = 128, PITCH = TOK + 8, NCB = 5, D = 128;
  constexpr int VPT = (TOK / 16) * 4 / 4;
  __shared__ __align__(16) __bf16 ft[128][PITCH];
  __shared__ __align__(16) __bf16 vt[128][PITCH];
  __shared__ __align__(16) __bf16 et[2][PITCH];
  const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % a.H;
  const int nbs = a.WB / 128, as = blockIdx.z / nbs, bs = blockIdx.z % nbs;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int AB = a.WA / 32, BB = a.WB / 32;
  const LinearMap lmap(BSRC == 1 ? a.R : 0, a.G);
  f32x16 acc[NCB];
#pragma unroll
  for (int i = 0; i < NCB; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[i][x] = 0.f;
  const int tf = w * 32 + r;
  int fcol[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) fcol[q] = (4 * g) * PITCH + ((((tf >> 3) ^ (2 * q)) << 3) | (tf & 7));
  const int vsw = (lane >> 4) << 1;
  const int vrow0 = 8 * (lane >> 4) * PITCH;
  const int rsw = ((r >> 3) & 3) << 1;
  __bf16 *ftp = &ft[0][0];
  __bf16 *vtp = &vt[0][0];
  const __bf16 one = static_cast<__bf16>(r == 0 ? 1.0f : 0.0f);
  const bf16x8 ones = bf16x8{one, one, one, one, one, one, one, one};
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  const int t_begin = chunk * a.CH, t_end = min(t_begin + a.CH, a.n_tok);
  for (int t0 = t_begin; t0 < t_end; t0 += TOK) {
    const int tb = t0 / 32 + w;
    const bool have = tb < a.n_tb;
    const bool valid = t0 + tf < a.n_tok;
    const int tok = lmap.token(min(t0 + tf, a.n_tok - 1));
    // A slab: four 32-row blocks of the image, scaled per token where asked for
    bf16x8 pa[4][2];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
      for (int s = 0; s < 2; ++s)
        pa[fb][s] = have ? a.a_img[((((int64_t)bh * a.n_tb + tb) * AB + 4 * as + fb) * 2 + s) * 64 + lane] : zero;
    if (a.a_scale) {
      const float sc = valid ? a.a_scale[(int64_t)bh * a.N + tok] : 0.f;
#pragma unroll
      for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          f32x8 t8;
#pragma unroll
          for (int i = 0; i < 8; ++i) t8[i] = static_cast<float>(pa[fb][s][i]) * sc;
          pa[fb][s] = __builtin_convertvector(t8, bf16x8);
        }
    }
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
      for (int x = 0; x < 16; ++x) ftp[(32 * fb + 8 * (x >> 2) + (x & 3)) * PITCH + fcol[x >> 2]] = pa[fb][x >> 3][x & 7];
    // B slab
    if constexpr (BSRC == 0) {
      bf16x8 pb[4][2];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int s = 0; s < 2; ++s)
          pb[cb][s] = have ? a.b_img[((((int64_t)bh * a.n_tb + tb) * BB + 4 * bs + cb) * 2 + s) * 64 + lane] : zero;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int x = 0; x < 16; ++x) vtp[(32 * cb + 8 * (x >> 2) + (x & 3)) * PITCH + fcol[x >> 2]] = pb[cb][x >> 3][x & 7];
    } else {
      // rows: pass p of wave w covers tokens 16 ((4 p + w) % 8) .. + 15 and the four 16-byte chunks 4 (p / 2) .. + 3
#pragma unroll
      for (int p = 0; p < VPT; ++p) {
        const int trow = 16 * ((4 * p + w) & 7) + (lane & 15), c8 = 4 * (p >> 1) + (lane >> 4);
        const int tk = lmap.token(min(t0 + trow, a.n_tok - 1));
        bf16x8 v8;
        if constexpr (BSRC == 1) v8 = load8<F32>(a.b_rows, base + (int64_t)tk * a.sn + c8 * 8);
        else v8 = static_cast<const bf16x8 *>(a.b_rows)[((int64_t)bh * a.N + tk) * (D / 8) + c8];
        const int col = (((trow >> 3) ^ vsw) << 3) | (trow & 7);
#pragma unroll
        for (int i = 0; i < 8; ++i) vtp[(32 * (p >> 1) + i) * PITCH + vrow0 + col] = v8[i];
      }
    }
    if (a.wcol && g == 0) {
      const float wv = a.wcol[(int64_t)bh * a.N + tok];
      const __bf16 whi = static_cast<__bf16>(wv);
      et[0][tf] = whi;
      et[1][tf] = static_cast<__bf16>(wv - static_cast<float>(whi));
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < TOK / 16; ++ks) {
      const int col = ((2 * ks + g) ^ rsw) << 3;
      const bf16x8 af = *reinterpret_cast<const bf16x8 *>(&ftp[(32 * w + r) * PITCH + col]);
      bf16x8 ex = ones;
      if (a.wcol) {
        const bf16x8 e8 = *reinterpret_cast<const bf16x8 *>(&et[r & 1][(2 * ks + g) << 3]);
        ex = r < 2 ? e8 : zero;
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const bf16x8 bfr = cb < 4 ? *reinterpret_cast<const bf16x8 *>(&vtp[(32 * cb + r) * PITCH + col]) : ex;
        acc[cb] = mfma32(af, bfr, acc[cb]);
      }
    }
    __syncthreads();
  }
  float *dst = a.part + ((((int64_t)bh * gridDim.x + chunk) * gridDim.z + blockIdx.z) * 4 + w) * NCB * 1024;
#pragma unroll
  for (int i = 0; i < NCB; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) dst[i * 1024 + x * 64 + lane] = acc[i][x];
}

// ------------------------------------------------------------------------------------------------
// wide_grad_reduce_kernel: grid (ceil(WA * (WB + 32) / 256), n_out).  Output o sums the partial tiles over the chunks of
// (batch b, head o) for every b (n_sum = B) or of (batch, head) pair o alone (n_sum = 1), in a fixed order.
// mat[o][row][col] row-major [WA][WB]; vec[o][row] = columns 0 + 1 of the extra block of B slab 0 (the hi and lo parts
// of a weighted sum, or the plain sum and zero).
__global__ __launch_bounds__(256) void wide_grad_reduce_kernel(const float *__restrict__ part, float *__restrict__ mat,
                                                               float *__restrict__ vec, int WA, int WB, int n_chunks, int n_sum,
                                                               int stride_sum) {
  const int o = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int cols = WB + 32;                         // the extra block as columns WB .. WB + 31
  if (e >= WA * cols) return;
  const int row = e / cols, col = e % cols;
  if (col > WB) return;                             // column WB also takes in column WB + 1
  const int nbs = WB / 128, nslab = (WA / 128) * nbs;
  const int as = row / 128, rb = (row % 128) / 32, rr = row % 32;
  const int bs = col < WB ? col / 128 : 0, cb = col < WB ? (col % 128) / 32 : 4, cc = col % 32;
  // row rr of a C tile sits in register x of lane group gg with crow(x, gg) = rr
  const int gg = (rr >> 2) & 1, x = 4 * (rr >> 3) + (rr & 3);
  const int64_t off = ((((int64_t)(as * nbs + bs)) * 4 + rb) * 5 + cb) * 1024 + x * 64 + gg * 32 + cc;
  float sum = 0.f;
  for (int b = 0; b < n_sum; ++b) {
    const int64_t bh = (int64_t)b * stride_sum + o;
    // four chunks per step: the loads of a step do not depend on each other (a plain running sum exposes one memory
    // round trip per chunk); the order of the additions is the same as one chunk at a time
    const int64_t cstride = (int64_t)nslab * 20 * 1024;
    const float *src0 = part + (bh * n_chunks) * cstride + off;
    const bool two = col == WB;
    int c = 0;
    for (; c + 4 <= n_chunks; c += 4) {
      float v[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = src0[(c + i) * cstride];
        u[i] = two ? src0[(c + i) * cstride + 1] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sum += v[i];
        if (two) sum += u[i];
      }
    }
    for (; c < n_chunks; ++c) {
      sum += src0[c * cstride];
      if (two) sum += src0[c * cstride + 1];
    }
  }
  if (col < WB) mat[((int64_t)o * WA + row) * WB + col] = sum;
  else vec[(int64_t)o * WA + row] = sum;
}

// ------------------------------------------------------------------------------------------------
// host side

template <typename T>
static inline T *ws_ptr(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }
static inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

void make_wide_grad_plan(const Plan &pl, const WidePlan &wp, size_t base_off, WideGradPlan &gp) {
  const size_t BH = (size_t)pl.B * pl.H;
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
  const size_t n_tb = wp.n_tb_q, nblk = (pl.F + 255) / 256;
  size_t off = base_off;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  const size_t KL = pl.DM > 0 ? pl.DM : pl.HD;                         // input width of the last layer
  gp.off_wt = take((size_t)pl.H * pl.F * KL * 2);
  gp.off_wtm = take((size_t)pl.H * pl.DM * pl.HD * 2);
  gp.off_shi = take(BH * pl.F * pl.D * 2);
  gp.off_slo = take(BH * pl.F * pl.D * 2);
  gp.off_dS = take(BH * pl.F * pl.D * 4);
  gp.off_dz = take(BH * pl.F * 4);
  gp.off_dshi = take(BH * pl.F * pl.D * 2);
  gp.off_dslo = take(BH * pl.F * pl.D * 2);
  gp.off_gsign = take(BH * pl.N * pl.D * 2);
  gp.off_rs = take(BH * pl.N * 4);
  gp.off_wp = take(BH * pl.N * 4);
  gp.off_tdt = take(BH * n_tb * 32 * (size_t)pl.F * 4);
  gp.off_pdot = take(BH * n_tb * nblk * 64 * 4);
  gp.off_du = take(BH * n_tb * 32 * (size_t)pl.F * 2);
  gp.off_dpre = take(BH * n_tb * 32 * (size_t)pl.HD * 2);
  gp.off_dpre2 = take(BH * n_tb * 32 * (size_t)pl.DM * 2);
  size_t slabs = (size_t)(pl.F / 128) * (KL / 128);                    // the largest product: the last layer's or the middle layer's
  if ((size_t)(pl.DM / 128) * (pl.HD / 128) > slabs) slabs = (size_t)(pl.DM / 128) * (pl.HD / 128);
  const int nc = gp.n_chunks_q > gp.n_chunks_k ? gp.n_chunks_q : gp.n_chunks_k;
  gp.off_part = take(BH * nc * slabs * 20 * 1024 * 4);
  gp.total = off;
}

// One product sum_tokens A^T [B | extra] and its reduction.  n_out = H (sum over the batch) or B*H.
template <int BSRC>
static hipError_t contract_and_reduce(const Plan &pl, ContractArgs c, int n_chunks, bool per_head, float *mat, float *vec,
                                      hipStream_t st) {
  const int BH = pl.B * pl.H;
  dim3 grid(n_chunks, BH, (c.WA / 128) * (c.WB / 128));
  if (pl.f32) wide_contract_kernel<BSRC, true><<<grid, 256, 0, st>>>(c);
  else wide_contract_kernel<BSRC, false><<<grid, 256, 0, st>>>(c);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 rgrid((c.WA * (c.WB + 32) + 255) / 256, per_head ? pl.H : BH);
  wide_grad_reduce_kernel<<<rgrid, 256, 0, st>>>(c.part, mat, vec, c.WA, c.WB, n_chunks, per_head ? pl.B : 1, per_head ? pl.H : 0);
  return hipGetLastError();
}

// Everything after the student's forward, for maps of any supported width and depth: S, z are in the forward's
// workspace region, y_teacher, y_student and row_den hold the two outputs and the student's row denominators.
hipError_t launch_wide_value_distill_backward(const Plan &pl, const WidePlan &wp, const WideGradPlan &gp, const void *q,
                                              const void *k, const void *v, const ha_feature_map &phi_q,
                                              const ha_feature_map &phi_k, const void *y_teacher, const void *y_student,
                                              const float *row_den, const ha_feature_map_grad &gq, const ha_feature_map_grad &gk,
                                              void *ws, hipStream_t st, double *l1_partial, double *loss) {
  const int BH = pl.B * pl.H, D = pl.D, F = pl.F, HD = pl.HD, DM = pl.DM, KL = DM > 0 ? DM : HD;
  hipError_t e;
  if ((e = launch_vd_rows(pl, y_teacher, y_student, row_den, ws_ptr<void>(ws, gp.off_gsign), ws_ptr<float>(ws, gp.off_rs),
                          ws_ptr<float>(ws, gp.off_wp), st, l1_partial, loss)) != hipSuccess)
    return e;
  if ((e = launch_natural_frags(ws_ptr<float>(ws, pl.off_S), ws_ptr<void>(ws, gp.off_shi), ws_ptr<void>(ws, gp.off_slo), F, D, BH,
                                st)) != hipSuccess)
    return e;
  for (int side = 0; side < 2; ++side) {
    const bool is_query = side == 0;
    const ha_feature_map &fm = is_query ? phi_q : phi_k;
    const ha_feature_map_grad &gm = is_query ? gq : gk;
    const int n_tok = is_query ? pl.N : pl.NL, n_tb = is_query ? wp.n_tb_q : wp.n_tb_k;
    const int n_chunks = is_query ? gp.n_chunks_q : gp.n_chunks_k, CH = is_query ? gp.CHq : gp.CHk;
    // this side's forward passes: h (hi + lo), pre-activations, softmax maxima / sums (phi_q is formed below)
    if ((e = launch_wide_map(pl, wp, is_query ? q : k, fm, is_query, ws, st)) != hipSuccess) return e;
    {
      dim3 grid((F * KL + 255) / 256, pl.H);
      if (pl.f32) wide_prep_t_kernel<true><<<grid, 256, 0, st>>>(fm.w2, ws_ptr<__bf16>(ws, gp.off_wt), F, KL);
      else wide_prep_t_kernel<false><<<grid, 256, 0, st>>>(fm.w2, ws_ptr<__bf16>(ws, gp.off_wt), F, KL);
      if ((e = hipGetLastError()) != hipSuccess) return e;
      if (DM > 0) {
        dim3 gridm((DM * HD + 255) / 256, pl.H);
        if (pl.f32) wide_prep_t_kernel<true><<<gridm, 256, 0, st>>>(fm.w_mid, ws_ptr<__bf16>(ws, gp.off_wtm), DM, HD);
        else wide_prep_t_kernel<false><<<gridm, 256, 0, st>>>(fm.w_mid, ws_ptr<__bf16>(ws, gp.off_wtm), DM, HD);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
    }
    WideGradArgs a;
    a.x = is_query ? q : k;
    a.u = is_query ? ws_ptr<void>(ws, gp.off_gsign) : v;
    a.rs = ws_ptr<float>(ws, gp.off_rs); a.wp = ws_ptr<float>(ws, gp.off_wp);
    a.m_hi = ws_ptr<bf16x8>(ws, is_query ? gp.off_shi : gp.off_dshi);
    a.m_lo = ws_ptr<bf16x8>(ws, is_query ? gp.off_slo : gp.off_dslo);
    a.zvec = is_query ? ws_ptr<float>(ws, pl.off_z) : ws_ptr<float>(ws, gp.off_dz);
    a.t_img = ws_ptr<f32x4>(ws, wp.off_u); a.tdt_img = ws_ptr<f32x4>(ws, gp.off_tdt);
    a.stat = ws_ptr<float>(ws, wp.off_stat); a.pdot = ws_ptr<float>(ws, gp.off_pdot);
    a.du_img = ws_ptr<bf16x8>(ws, gp.off_du); a.phi_img = ws_ptr<bf16x8>(ws, wp.off_phi);
    a.H = pl.H; a.N = pl.N; a.F = F; a.n_tok = n_tok; a.n_tb = n_tb; a.R = pl.R; a.G = pl.G; a.P = pl.P;
    a.act = is_query ? pl.act_q : pl.act_k;
    const bool fused = a.act != 0 || F <= 256;       // the softmax Jacobian's sum stays inside one workgroup
    a.sb = pl.sb; a.sh = pl.sh; a.sn = pl.sn;
    {
      dim3 grid((n_tb + 3) / 4, (F + 255) / 256, BH);
#define HA_DPHI(F32, QUERY)                                                      \
  do {                                                                          \
    if (fused) wide_dphi_kernel<128, F32, QUERY, true><<<grid, 256, 0, st>>>(a); \
    else wide_dphi_kernel<128, F32, QUERY, false><<<grid, 256, 0, st>>>(a);      \
  } while (0)
      if (is_query) { if (pl.f32) HA_DPHI(true, true); else HA_DPHI(false, true); }
      else { if (pl.f32) HA_DPHI(true, false); else HA_DPHI(false, false); }
#undef HA_DPHI
      if ((e = hipGetLastError()) != hipSuccess) return e;
      if (!fused) {
        dim3 grid2((n_tb + 3) / 4, BH);
        wide_du_kernel<<<grid2, 256, 0, st>>>(a.t_img, a.tdt_img, a.pdot, ws_ptr<bf16x8>(ws, gp.off_du), F, n_tb, a.act);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
      // back through the last layer (and the middle one): dpre = (W^T d) [h > 0]
      const bf16x8 *d_in = ws_ptr<bf16x8>(ws, gp.off_du);
      if (DM > 0) {
        dim3 grid3((n_tb + 3) / 4, (DM + 255) / 256, BH);
        wide_back_layer_kernel<<<grid3, 256, 0, st>>>(d_in, ws_ptr<bf16x8>(ws, gp.off_wt), ws_ptr<bf16x8>(ws, wp.off_h2hi),
                                                      ws_ptr<bf16x8>(ws, gp.off_dpre2), pl.H, F, DM, n_tb);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        d_in = ws_ptr<bf16x8>(ws, gp.off_dpre2);
      }
      dim3 grid3((n_tb + 3) / 4, (HD + 255) / 256, BH);
      wide_back_layer_kernel<<<grid3, 256, 0, st>>>(d_in, ws_ptr<bf16x8>(ws, DM > 0 ? gp.off_wtm : gp.off_wt),
                                                    ws_ptr<bf16x8>(ws, wp.off_hhi), ws_ptr<bf16x8>(ws, gp.off_dpre), pl.H,
                                                    DM > 0 ? DM : F, HD, n_tb);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    ContractArgs c;
    c.a_scale = nullptr; c.b_img = nullptr; c.b_rows = nullptr; c.wcol = nullptr;
    c.part = ws_ptr<float>(ws, gp.off_part);
    c.H = pl.H; c.N = pl.N; c.n_tok = n_tok; c.n_tb = n_tb; c.R = is_query ? 0 : pl.R; c.G = pl.G; c.CH = CH;
    c.sb = pl.sb; c.sh = pl.sh; c.sn = pl.sn;
    // [dW2 | db2] = sum du [h | 1]^T, h the input of the last layer
    c.a_img = ws_ptr<bf16x8>(ws, gp.off_du); c.WA = F;
    c.b_img = ws_ptr<bf16x8>(ws, DM > 0 ? wp.off_h2hi : wp.off_hhi); c.WB = KL;
    if ((e = contract_and_reduce<0>(pl, c, n_chunks, true, gm.w2, gm.b2, st)) != hipSuccess) return e;
    if (DM > 0) {
      // [dW_mid | db_mid] = sum dpre2 [h1 | 1]^T
      c.a_img = ws_ptr<bf16x8>(ws, gp.off_dpre2); c.WA = DM;
      c.b_img = ws_ptr<bf16x8>(ws, wp.off_hhi); c.WB = HD;
      if ((e = contract_and_reduce<0>(pl, c, n_chunks, true, gm.w_mid, gm.b_mid, st)) != hipSuccess) return e;
    }
    // [dW1 | db1] = sum dpre [x | 1]^T
    c.a_img = ws_ptr<bf16x8>(ws, gp.off_dpre); c.WA = HD;
    c.b_img = nullptr; c.b_rows = is_query ? q : k; c.WB = D;
    if ((e = contract_and_reduce<1>(pl, c, n_chunks, true, gm.w1, gm.b1, st)) != hipSuccess) return e;
    if (is_query) {
      // [dS | dz] = sum (phi_q / den) [g | dden den]^T per (batch, head), then dS as operand fragments for the key side
      c.a_img = ws_ptr<bf16x8>(ws, wp.off_phi); c.WA = F;
      c.a_scale = ws_ptr<float>(ws, gp.off_rs);
      c.b_rows = ws_ptr<void>(ws, gp.off_gsign); c.WB = D;
      c.wcol = ws_ptr<float>(ws, gp.off_wp);
      if ((e = contract_and_reduce<2>(pl, c, n_chunks, false, ws_ptr<float>(ws, gp.off_dS), ws_ptr<float>(ws, gp.off_dz), st)) !=
          hipSuccess)
        return e;
      if ((e = launch_natural_frags(ws_ptr<float>(ws, gp.off_dS), ws_ptr<void>(ws, gp.off_dshi), ws_ptr<void>(ws, gp.off_dslo), F,
                                    D, BH, st)) != hipSuccess)
        return e;
    }
  }
  return hipSuccess;
}

}  // namespace ha
