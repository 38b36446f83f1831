// Feature maps of any width (Attention Surgery, Sec. 3.2 "Characterization of phi"; Tab. "phi": d -> P d -> P d
// for P = 2, 3, 4 and the three-layer P = 6 map), gfx950.  The fused kernels keep a token's hidden activations and
// all its output channels in registers, which ends at 256 channels.  Here every layer is a pass of its own and
// activations travel through HBM, in exactly the register image the next product wants:
//
//   wide_prep_kernel       one weight matrix -> A-operand fragments (natural order for layer 1, chained after it)
//   wide_layer1_kernel     h^T = relu(W1 x^T + b1)                     x from q / k, h as hi + lo bf16
//   wide_layer_kernel      h'^T = relu(W h^T + b)  or  u^T = W h^T + b  (last layer: fp32 pre-activations)
//   (output stage)         softmax / exp / relu over all channels of a token, slice powers, bf16: applied by the two
//                          consumers below while they read the pre-activations, so phi never visits HBM
//   wide_state_kernel      [S | z] += phi_k^T [V | 1], one 128-channel slab of S per workgroup
//   wide_lin_kernel        n_i = phi_q(q_i) S   (fp32, in the layout of the query kernel's accumulators), e_i = phi_q(q_i).z
// The query kernel then adds n_i and e_i in its epilogue instead of evaluating phi_q itself.
//
// Register images ("C image" of a 32-token block tb of (batch, head) bh; lane = 32 g + r owns token 32 tb + r):
//   activations   bf16x8 [bh][tb][W/32][2][64]   piece (block c, half s) = channels 32 c + crow(8 s + t, g), t = 0..7,
//                                                i.e. the B operand ("chained" order) of the next product
//   fp32 tiles    f32x4  [bh][tb][W/32][4][64]   piece (block c, quad x) = channels 32 c + crow(4 x + j, g), j = 0..3
#include "ha_device.h"
#include "ha_plan.h"

namespace ha {

struct WideArgs {
  const void *x;                 // layer 1: q or k (io dtype, strided)
  const bf16x8 *in_hi, *in_lo;   // later layers / consumers: activations of the previous pass
  const bf16x8 *wf;              // weight fragments of this layer, all heads
  const float *bias;             // [H][NOUT] or null
  bf16x8 *out_hi, *out_lo;       // hidden layers
  f32x4 *out_u;                  // last layer
  float *out_stat;               // last layer: [bh][tb][256-channel block][2][64] running maximum and sum of exponentials
  int H, K, NOUT, n_tok, n_tb, R, G;
  int64_t sb, sh, sn;
};

// ------------------------------------------------------------------------------------------------
// wide_prep_kernel: grid (ceil(NOUT*K / 256), H).  W [H][NOUT][K] (io dtype) ->
//   natural:  wf[h][ob][ks][lane][t]    = W[h][32 ob + r][16 ks + 8 g + t]
//   chained:  wf[h][ob][kb][s][lane][t] = W[h][32 ob + r][32 kb + crow(8 s + t, g)]
template <bool F32, bool CHAINED>
__global__ __launch_bounds__(256) void wide_prep_kernel(const void *__restrict__ wsrc, __bf16 *__restrict__ wf, int NOUT, int K) {
  const int h = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= NOUT * K) return;
  const int t = e & 7, lane = (e >> 3) & 63, rest = e >> 9;
  const int r = lane & 31, g = lane >> 5;
  int row, col;
  if constexpr (CHAINED) {
    const int KB = K / 32;
    const int s = rest & 1, kb = (rest >> 1) % KB, ob = (rest >> 1) / KB;
    row = 32 * ob + r;
    col = 32 * kb + crow(8 * s + t, g);
  } else {
    const int KS = K / 16;
    const int ks = rest % KS, ob = rest / KS;
    row = 32 * ob + r;
    col = 16 * ks + 8 * g + t;
  }
  const int64_t src = ((int64_t)h * NOUT + row) * K + col;
  float val;
  if constexpr (F32) val = static_cast<const float *>(wsrc)[src];
  else val = static_cast<float>(static_cast<const __bf16 *>(wsrc)[src]);
  wf[(int64_t)h * NOUT * K + e] = static_cast<__bf16>(val);
}

// ------------------------------------------------------------------------------------------------
// wide_layer1_kernel: grid (ceil(n_tb / 4), NOUT / 128, B*H), 4 waves, one 32-token block per wave and four
// 32-channel output blocks per workgroup row.  W1 fragments in natural order (weight_prep_kernel).
template <int D, bool F32>
__global__ __launch_bounds__(256) void wide_layer1_kernel(WideArgs a) {
  constexpr int KS = D / 16;
  const int bh = blockIdx.z, h = bh % a.H;
  const int lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
  const int tb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tb >= a.n_tb) return;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const LinearMap lmap(a.R, a.G);
  const int tok = lmap.token(min(32 * tb + r, a.n_tok - 1));
  bf16x8 xf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) xf[ks] = load8<F32>(a.x, base + (int64_t)tok * a.sn + 16 * ks + 8 * g);
  const GlobalFrags wf = global_frags(a.wf + (int64_t)h * (a.NOUT * D / 8), a.NOUT * D * 2);
  const int HB = a.NOUT / 32;
  for (int j = 0; j < 4; ++j) {
    const int hb = blockIdx.y * 4 + j;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = a.bias ? a.bias[(int64_t)h * a.NOUT + 32 * hb + crow(v, g)] : 0.f;
    bf16x8 w8[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) w8[ks] = frag_at(wf, hb * KS + ks, lane);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc = mfma32(w8[ks], xf[ks], acc);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      f32x8 t, lo;
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = fmaxf(acc[8 * s + i], 0.f);
      const bf16x8 hi = __builtin_convertvector(t, bf16x8);
#pragma unroll
      for (int i = 0; i < 8; ++i) lo[i] = t[i] - static_cast<float>(hi[i]);
      const int64_t o = ((((int64_t)bh * a.n_tb + tb) * HB + hb) * 2 + s) * 64 + lane;
      a.out_hi[o] = hi;
      a.out_lo[o] = __builtin_convertvector(lo, bf16x8);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// wide_layer_kernel: grid (ceil(n_tb / 4), ceil(NOUT / 256), B*H), 4 waves.  Input activations as hi + lo C images
// (width K), weights [NOUT x K] as fragments in chained order.  LAST: fp32 pre-activations out; otherwise relu
// and hi + lo bf16.  Every wave owns one 32-token block and all (up to eight) 32-channel output tiles of the
// workgroup, so an activation fragment is read once per 256 output channels; the weight fragments are the same
// for the four waves and pass through LDS, two 32-channel input blocks per stage, the next stage in flight
// (direct-to-LDS) while the 64 matrix instructions of the current one run.
// FULL: NOUT is a multiple of 256, every workgroup has all eight output tiles: the inner loops carry no tile-count
// tests, so the weight fragments of a half step are requested together ahead of their matrix instructions.
template <bool LAST, bool FULL>
__global__ __launch_bounds__(256, 2) void wide_layer_kernel(WideArgs a) {
  constexpr int NT = 8, KCH = 2, STG = NT * KCH * 2 * 64;       // bf16x8 per stage buffer (32 KiB)
  __shared__ bf16x8 wl[2][STG];
  const int bh = blockIdx.z, h = bh % a.H;
  const int lane = threadIdx.x & 63, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool live = blockIdx.x * 4 + w < a.n_tb;                 // idle waves keep staging and synchronising
  const int tb = live ? blockIdx.x * 4 + w : a.n_tb - 1;
  const int KB = a.K / 32, OB = a.NOUT / 32;
  const int ob0 = blockIdx.y * NT;
  const int nt = FULL ? NT : min(NT, OB - ob0);
  const bf16x8 *wg = a.wf + (int64_t)h * ((int64_t)a.NOUT * a.K / 8);
  const bf16x8 *bhi = a.in_hi + ((int64_t)bh * a.n_tb + tb) * KB * 128 + lane;
  const bf16x8 *blo = a.in_lo + ((int64_t)bh * a.n_tb + tb) * KB * 128 + lane;
  f32x16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = (a.bias && j < nt) ? a.bias[(int64_t)h * a.NOUT + 32 * (ob0 + j) + crow(v, g)] : 0.f;
  auto stage = [&](int c, int buf) {              // input blocks c KCH .. c KCH + KCH - 1 of every output tile
    for (int j = 0; j < nt; ++j)
      dma_to_lds(wg + (((int64_t)(ob0 + j) * KB + c * KCH) * 2) * 64, &wl[buf][j * KCH * 2 * 64], KCH * 2, w, 4, lane);
  };
  bf16x8 cb_hi[2], cb_lo[2], nb_hi[2], nb_lo[2];
  auto request_b = [&](int kb, bf16x8 (&hi)[2], bf16x8 (&lo)[2]) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      hi[s] = bhi[(kb * 2 + s) * 64];
      lo[s] = blo[(kb * 2 + s) * 64];
    }
  };
  stage(0, 0);
  request_b(0, cb_hi, cb_lo);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  const int n_stages = KB / KCH;
  for (int c = 0; c < n_stages; ++c) {
    if (c + 1 < n_stages) stage(c + 1, (c + 1) & 1);
    const bf16x8 *wbuf = &wl[c & 1][lane];
#pragma unroll
    for (int kbl = 0; kbl < KCH; ++kbl) {
      const int kb = c * KCH + kbl;
      if (kb + 1 < KB) request_b(kb + 1, nb_hi, nb_lo);
      if constexpr (FULL) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int j0 = 0; j0 < NT; j0 += 4) {
            bf16x8 af[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) af[j] = wbuf[((j0 + j) * KCH * 2 + kbl * 2 + s) * 64];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              acc[j0 + j] = mfma32(af[j], cb_lo[s], acc[j0 + j]);
              acc[j0 + j] = mfma32(af[j], cb_hi[s], acc[j0 + j]);
            }
          }
      } else {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            if (j < nt) {
              const bf16x8 af = wbuf[(j * KCH * 2 + kbl * 2 + s) * 64];
              acc[j] = mfma32(af, cb_lo[s], acc[j]);
              acc[j] = mfma32(af, cb_hi[s], acc[j]);
            }
      }
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        cb_hi[s] = nb_hi[s];
        cb_lo[s] = nb_lo[s];
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                               // the next stage has landed; this one may be overwritten
  }
  if (!live) return;
  if constexpr (LAST) {
    // per token: maximum of this workgroup's channels and the sum of exponentials against it, so that the output
    // stage can form the softmax over all channels with a single sweep over the pre-activations
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < NT; ++j)
      if (j < nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, acc[j][v]);
    m = xhalf_max(m);
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NT; ++j)
      if (j < nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += fast_exp2((acc[j][v] - m) * kLog2e);
    sum = xhalf_sum(sum);
    float *st = a.out_stat + ((((int64_t)bh * a.n_tb + tb) * gridDim.y + blockIdx.y) * 2) * 64 + lane;
    st[0] = m;
    st[64] = sum;
  }
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    if (j >= nt) break;
    const int64_t blk = ((int64_t)bh * a.n_tb + tb) * OB + ob0 + j;
    if constexpr (LAST) {
#pragma unroll
      for (int x4 = 0; x4 < 4; ++x4)
        a.out_u[(blk * 4 + x4) * 64 + lane] = f32x4{acc[j][4 * x4], acc[j][4 * x4 + 1], acc[j][4 * x4 + 2], acc[j][4 * x4 + 3]};
    } else {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        f32x8 t, lo;
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = fmaxf(acc[j][8 * s + i], 0.f);
        const bf16x8 hi = __builtin_convertvector(t, bf16x8);
#pragma unroll
        for (int i = 0; i < 8; ++i) lo[i] = t[i] - static_cast<float>(hi[i]);
        a.out_hi[(blk * 2 + s) * 64 + lane] = hi;
        a.out_lo[(blk * 2 + s) * 64 + lane] = __builtin_convertvector(lo, bf16x8);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Output stage of a feature map, applied by the consumers of phi while they read the fp32 pre-activations (so phi
// itself never visits HBM): normalisation (softmax: against the maximum and sum combined from the per-256-channel-block
// values the last layer left behind), slice powers, rounding.
constexpr int WIDE_FMAX = 768;

struct WideOutStage {
  float off, inv, inv_groups;     // softmax: exp2(u log2 e + off) * inv;  1 / (8-channel groups per slice)
  int act;
};

// One lane's view (token 32 tb + lane % 32) of the softmax statistics of its token.
static __device__ __forceinline__ WideOutStage wide_out_stage(const float *__restrict__ stat, int64_t bh_tb, int F, int act,
                                                              int P, int lane) {
  WideOutStage o;
  o.off = 0.f; o.inv = 1.f; o.act = act;
  o.inv_groups = 8.0f * (float)P / (float)F;
  if (act == 0) {
    const int nblk = (F + 255) / 256;
    const float *st = stat + (bh_tb * nblk * 2) * 64 + lane;
    float m = -INFINITY;
    for (int b = 0; b < nblk; ++b) m = fmaxf(m, st[b * 128]);
    float sum = 0.f;
    for (int b = 0; b < nblk; ++b) sum += st[b * 128 + 64] * fast_exp2((st[b * 128] - m) * kLog2e);
    o.off = -m * kLog2e;
    o.inv = 1.0f / sum;
  }
  return o;
}

// phi of the 32-channel tile fb of one token block from its fp32 C image piece: the two bf16 pieces (chained order)
// the next product takes as its B operand; zero for tokens past the end.
static __device__ __forceinline__ void wide_phi_tile(const f32x4 (&raw)[4], int fb, const WideOutStage &o, bool valid,
                                                     bf16x8 (&out)[2]) {
  f32x16 u;
#pragma unroll
  for (int x4 = 0; x4 < 4; ++x4)
#pragma unroll
    for (int j = 0; j < 4; ++j) u[4 * x4 + j] = raw[x4][j];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    if (o.act == 0) u[v] = fast_exp2(__builtin_fmaf(u[v], kLog2e, o.off)) * o.inv;
    else if (o.act == 1) u[v] = fast_exp2(u[v] * kLog2e);
    else u[v] = fmaxf(u[v], 0.f);
  }
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    f32x8 t8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // slice power - 1 = (8-channel group index) / (groups per slice), wave-uniform; exact in fp32 for these sizes
      const int extra = (int)(((float)(4 * fb + 2 * s + i / 4) + 0.5f) * o.inv_groups);
      const float t0 = u[8 * s + i], t2 = t0 * t0;
      float t = (extra & 1) ? t2 : t0;                           // t0^(extra + 1), extra in 0..7
      t = (extra & 2) ? t * t2 : t;
      t = (extra & 4) ? t * (t2 * t2) : t;
      t8[i] = valid ? t : 0.f;
    }
    out[s] = __builtin_convertvector(t8, bf16x8);
  }
}
static __device__ __forceinline__ void wide_load_tile(const f32x4 *__restrict__ src, int fb, f32x4 (&raw)[4]) {
#pragma unroll
  for (int x4 = 0; x4 < 4; ++x4) raw[x4] = src[(fb * 4 + x4) * 64];
}
static __device__ __forceinline__ void wide_phi_tile(const f32x4 *__restrict__ src, int fb, const WideOutStage &o, bool valid,
                                                     bf16x8 (&out)[2]) {
  f32x4 raw[4];
  wide_load_tile(src, fb, raw);
  wide_phi_tile(raw, fb, o, valid, out);
}

// ------------------------------------------------------------------------------------------------
// wide_state_kernel: grid (n_chunks, B*H, F / 128), 4 waves.  As the contraction half of state_kernel, with
// phi_k formed from the fp32 pre-activations of the last layer as they are read; workgroup z owns feature rows
// 128 z .. 128 z + 127 of [S | z], wave w row block w of those.  Partial tiles go where state_kernel puts them
// (part[bh][chunk][row block * NCB + column block][v][lane]), so state_reduce_kernel serves both.
template <int D, bool F32>
__global__ __launch_bounds__(256, 1) void wide_state_kernel(const f32x4 *__restrict__ u_img, const float *__restrict__ stat,
                                                            const void *__restrict__ v, float *__restrict__ part, int H,
                                                            int NL, int R, int G, int CH, int F, int n_tb, int act, int P,
                                                            int64_t sb, int64_t sh, int64_t sn) {
  constexpr int TOK = 128, PITCH = TOK + 8, NCB = D / 32 + 1;
  constexpr int CG = D / 32, VPT = (TOK / 16) * CG / 4;
  __shared__ __align__(16) __bf16 ft[128][PITCH];
  __shared__ __align__(16) __bf16 vt[D][PITCH];
  const int chunk = blockIdx.x, bh = blockIdx.y, zb = blockIdx.z, h = bh % H;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)h * sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int FB = F / 32;
  const LinearMap lmap(R, G);
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
  const int lt_begin = chunk * CH, lt_end = min(lt_begin + CH, NL);
  for (int t0 = lt_begin; t0 < lt_end; t0 += TOK) {
    bf16x8 vreg[VPT];
#pragma unroll
    for (int p = 0; p < VPT; ++p) {
      const int trow = 16 * ((4 * p + w) & 7) + (lane & 15), c8 = 4 * (p >> 1) + (lane >> 4);
      const int tok = lmap.token(min(t0 + trow, NL - 1));
      vreg[p] = load8<F32>(v, base + (int64_t)tok * sn + c8 * 8);
    }
    const int tb = min(t0 / 32 + w, n_tb - 1);            // blocks past the end: clamped, their tokens are not valid
    const bool valid = t0 + tf < NL;
    const WideOutStage os = wide_out_stage(stat, (int64_t)bh * n_tb + tb, F, act, P, lane);
    const f32x4 *usrc = u_img + ((int64_t)bh * n_tb + tb) * FB * 256 + lane;
    bf16x8 ph[4][2];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) wide_phi_tile(usrc, 4 * zb + fb, os, valid, ph[fb]);
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
      for (int x = 0; x < 16; ++x) ftp[(32 * fb + 8 * (x >> 2) + (x & 3)) * PITCH + fcol[x >> 2]] = ph[fb][x >> 3][x & 7];
#pragma unroll
    for (int p = 0; p < VPT; ++p) {
      const int trow = 16 * ((4 * p + w) & 7) + (lane & 15);
      const int col = (((trow >> 3) ^ vsw) << 3) | (trow & 7);
#pragma unroll
      for (int i = 0; i < 8; ++i) vtp[(32 * (p >> 1) + i) * PITCH + vrow0 + col] = vreg[p][i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < TOK / 16; ++ks) {
      const int col = ((2 * ks + g) ^ rsw) << 3;
      const bf16x8 af = *reinterpret_cast<const bf16x8 *>(&ftp[(32 * w + r) * PITCH + col]);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const bf16x8 bfr = cb < D / 32 ? *reinterpret_cast<const bf16x8 *>(&vtp[(32 * cb + r) * PITCH + col]) : ones;
        acc[cb] = mfma32(af, bfr, acc[cb]);
      }
    }
    __syncthreads();
  }
  float *dst = part + (((int64_t)bh * gridDim.x + chunk) * FB + 4 * zb + w) * NCB * 1024;
#pragma unroll
  for (int i = 0; i < NCB; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) dst[i * 1024 + x * 64 + lane] = acc[i][x];
}

// ------------------------------------------------------------------------------------------------
// wide_lin_kernel: grid (ceil(n_tb / 4), B*H).  Output stage of phi_q and the linear part of Eq. "hybrid" per 32-query
// block: n^T = S^T phi_q^T (A operand = S^T as hi + lo fragments in chained order, state_reduce_kernel's layout; B
// operand = phi_q, formed tile by tile from the fp32 pre-activations) and e = phi_q . z with the rounded phi_q, as the
// numerator uses it.  Output: n as an fp32 C image of width D, i.e. the layout of the query kernel's accumulators;
// e[bh][token].
template <int D>
__global__ __launch_bounds__(256) void wide_lin_kernel(const f32x4 *__restrict__ u_img, const float *__restrict__ stat,
                                                       const bf16x8 *__restrict__ st_hi, const bf16x8 *__restrict__ st_lo,
                                                       const float *__restrict__ z, f32x4 *__restrict__ lin,
                                                       float *__restrict__ e_out, int F, int n_tok, int n_tb, int act, int P) {
  constexpr int RB = D / 32;
  __shared__ float zl[WIDE_FMAX];
  const int bh = blockIdx.y;
  for (int i = threadIdx.x; i < F; i += 256) zl[i] = z[(int64_t)bh * F + i];
  __syncthreads();
  const int lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
  const int tb = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tb >= n_tb) return;
  const int FB = F / 32;
  const bool valid = 32 * tb + r < n_tok;
  const WideOutStage os = wide_out_stage(stat, (int64_t)bh * n_tb + tb, F, act, P, lane);
  const f32x4 *usrc = u_img + ((int64_t)bh * n_tb + tb) * FB * 256 + lane;
  const GlobalFrags shi = global_frags(st_hi + (int64_t)bh * (D * F / 8), D * F * 2);
  const GlobalFrags slo = global_frags(st_lo + (int64_t)bh * (D * F / 8), D * F * 2);
  f32x16 acc[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
  float dot = 0.f;
  for (int fb = 0; fb < FB; ++fb) {
    bf16x8 b[2], ahi[RB][2], alo[RB][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        ahi[rb][s] = frag_at(shi, (rb * FB + fb) * 2 + s, lane);
        alo[rb][s] = frag_at(slo, (rb * FB + fb) * 2 + s, lane);
      }
    wide_phi_tile(usrc, fb, os, valid, b);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int i = 0; i < 8; ++i) dot += static_cast<float>(b[s][i]) * zl[32 * fb + crow(8 * s + i, g)];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        acc[rb] = mfma32(alo[rb][s], b[s], acc[rb]);
        acc[rb] = mfma32(ahi[rb][s], b[s], acc[rb]);
      }
    }
  }
  dot = xhalf_sum(dot);
  if (g == 0 && valid) e_out[(int64_t)bh * n_tok + 32 * tb + r] = dot;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int x4 = 0; x4 < 4; ++x4)
      lin[((((int64_t)bh * n_tb + tb) * RB + rb) * 4 + x4) * 64 + lane] =
          f32x4{acc[rb][4 * x4], acc[rb][4 * x4 + 1], acc[rb][4 * x4 + 2], acc[rb][4 * x4 + 3]};
}

// ------------------------------------------------------------------------------------------------
// host side

template <typename T>
static inline T *ws_ptr(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }
static inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

void make_wide_plan(const Plan &pl, size_t base_off, WidePlan &wp) {
  const size_t BH = (size_t)pl.B * pl.H;
  wp.n_tb_q = (pl.N + 31) / 32;
  wp.n_tb_k = (pl.NL + 31) / 32;
  const size_t n_tb = wp.n_tb_q;                      // the key side (fewer tokens) reuses the query side's buffers
  size_t off = base_off;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  const int KL = pl.DM > 0 ? pl.DM : pl.HD;            // input width of the last layer
  wp.off_w1 = take((size_t)pl.H * pl.HD * pl.D * 2);
  wp.off_wm = take((size_t)pl.H * pl.DM * pl.HD * 2);
  wp.off_w2 = take((size_t)pl.H * pl.F * KL * 2);
  wp.off_hhi = take(BH * n_tb * 32 * pl.HD * 2);
  wp.off_hlo = take(BH * n_tb * 32 * pl.HD * 2);
  wp.off_h2hi = take(BH * n_tb * 32 * pl.DM * 2);
  wp.off_h2lo = take(BH * n_tb * 32 * pl.DM * 2);
  wp.off_u = take(BH * n_tb * 32 * (size_t)pl.F * 4);
  wp.off_stat = take(BH * n_tb * ((pl.F + 255) / 256) * 2 * 64 * sizeof(float));
  wp.off_phi = take(BH * n_tb * 32 * (size_t)pl.F * 2);
  wp.off_lin = take(BH * n_tb * 32 * (size_t)pl.D * 4);
  wp.off_e = take(BH * (size_t)pl.N * 4);
  wp.total = off;
}

// One feature map over one token set: weight fragments, layer 1, (middle layer,) last layer, which leaves the fp32
// pre-activations and the softmax statistics; the output stage belongs to whoever reads them next.  is_query: all N
// tokens of q; otherwise the linear tokens of k.
hipError_t launch_wide_map(const Plan &pl, const WidePlan &wp, const void *x, const ha_feature_map &fm, bool is_query,
                           void *ws, hipStream_t st) {
  const int BH = pl.B * pl.H;
  const int n_tok = is_query ? pl.N : pl.NL, n_tb = is_query ? wp.n_tb_q : wp.n_tb_k;
  hipError_t e;
  const int KL = pl.DM > 0 ? pl.DM : pl.HD;
  // weight fragments of this map
  {
    auto prep = [&](const void *wsrc, size_t off, int nout, int kdim, bool chained) {
      dim3 grid((nout * kdim + 255) / 256, pl.H);
      __bf16 *dst = ws_ptr<__bf16>(ws, off);
      if (pl.f32) {
        if (chained) wide_prep_kernel<true, true><<<grid, 256, 0, st>>>(wsrc, dst, nout, kdim);
        else wide_prep_kernel<true, false><<<grid, 256, 0, st>>>(wsrc, dst, nout, kdim);
      } else {
        if (chained) wide_prep_kernel<false, true><<<grid, 256, 0, st>>>(wsrc, dst, nout, kdim);
        else wide_prep_kernel<false, false><<<grid, 256, 0, st>>>(wsrc, dst, nout, kdim);
      }
    };
    prep(fm.w1, wp.off_w1, pl.HD, pl.D, false);
    if (pl.DM > 0) prep(fm.w_mid, wp.off_wm, pl.DM, pl.HD, true);
    prep(fm.w2, wp.off_w2, pl.F, KL, true);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  WideArgs a;
  a.x = x;
  a.H = pl.H; a.n_tok = n_tok; a.n_tb = n_tb; a.R = is_query ? 0 : pl.R; a.G = pl.G;
  a.sb = pl.sb; a.sh = pl.sh; a.sn = pl.sn;
  a.in_hi = a.in_lo = nullptr;
  a.out_u = nullptr;
  a.out_stat = nullptr;
  // layer 1: d -> HD
  a.wf = ws_ptr<bf16x8>(ws, wp.off_w1);
  a.bias = fm.b1; a.K = pl.D; a.NOUT = pl.HD;
  a.out_hi = ws_ptr<bf16x8>(ws, wp.off_hhi); a.out_lo = ws_ptr<bf16x8>(ws, wp.off_hlo);
  {
    dim3 grid((n_tb + 3) / 4, pl.HD / 128, BH);
    if (pl.f32) wide_layer1_kernel<128, true><<<grid, 256, 0, st>>>(a);
    else wide_layer1_kernel<128, false><<<grid, 256, 0, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  a.in_hi = ws_ptr<bf16x8>(ws, wp.off_hhi); a.in_lo = ws_ptr<bf16x8>(ws, wp.off_hlo);
  if (pl.DM > 0) {
    // middle layer of a three-layer map: HD -> DM, relu, hi + lo
    a.wf = ws_ptr<bf16x8>(ws, wp.off_wm);
    a.bias = fm.b_mid; a.K = pl.HD; a.NOUT = pl.DM;
    a.out_hi = ws_ptr<bf16x8>(ws, wp.off_h2hi); a.out_lo = ws_ptr<bf16x8>(ws, wp.off_h2lo);
    dim3 grid((n_tb + 3) / 4, (pl.DM + 255) / 256, BH);
    if (pl.DM % 256 == 0) wide_layer_kernel<false, true><<<grid, 256, 0, st>>>(a);
    else wide_layer_kernel<false, false><<<grid, 256, 0, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    a.in_hi = ws_ptr<bf16x8>(ws, wp.off_h2hi); a.in_lo = ws_ptr<bf16x8>(ws, wp.off_h2lo);
  }
  // last layer: -> F, fp32 pre-activations
  a.wf = ws_ptr<bf16x8>(ws, wp.off_w2);
  a.bias = fm.b2; a.K = KL; a.NOUT = pl.F;
  a.out_hi = a.out_lo = nullptr;
  a.out_u = ws_ptr<f32x4>(ws, wp.off_u);
  a.out_stat = ws_ptr<float>(ws, wp.off_stat);
  {
    dim3 grid((n_tb + 3) / 4, (pl.F + 255) / 256, BH);
    if (pl.F % 256 == 0) wide_layer_kernel<true, true><<<grid, 256, 0, st>>>(a);
    else wide_layer_kernel<true, false><<<grid, 256, 0, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

// Key side: phi_k over the linear tokens, then [S | z] (partials + the forward's reduction).
hipError_t launch_wide_key_side(const Plan &pl, const WidePlan &wp, const void *k, const void *v, const ha_feature_map &phi_k,
                                void *ws, hipStream_t st) {
  hipError_t e = launch_wide_map(pl, wp, k, phi_k, false, ws, st);
  if (e != hipSuccess) return e;
  dim3 grid(pl.n_chunks, pl.B * pl.H, pl.F / 128);
  if (pl.f32)
    wide_state_kernel<128, true><<<grid, 256, 0, st>>>(ws_ptr<f32x4>(ws, wp.off_u), ws_ptr<float>(ws, wp.off_stat), v,
                                                       ws_ptr<float>(ws, pl.off_part), pl.H, pl.NL, pl.R, pl.G, pl.CH, pl.F,
                                                       wp.n_tb_k, pl.act_k, pl.P, pl.sb, pl.sh, pl.sn);
  else
    wide_state_kernel<128, false><<<grid, 256, 0, st>>>(ws_ptr<f32x4>(ws, wp.off_u), ws_ptr<float>(ws, wp.off_stat), v,
                                                        ws_ptr<float>(ws, pl.off_part), pl.H, pl.NL, pl.R, pl.G, pl.CH, pl.F,
                                                        wp.n_tb_k, pl.act_k, pl.P, pl.sb, pl.sh, pl.sn);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return launch_state_reduce(pl, ws, st);
}

// Query side: phi_q over all tokens, e = phi_q . z, n = phi_q S; the query kernel picks both up in its epilogue.
hipError_t launch_wide_query_side(const Plan &pl, const WidePlan &wp, const void *q, const ha_feature_map &phi_q, void *ws,
                                  hipStream_t st) {
  hipError_t e = launch_wide_map(pl, wp, q, phi_q, true, ws, st);
  if (e != hipSuccess) return e;
  dim3 grid((wp.n_tb_q + 3) / 4, pl.B * pl.H);
  wide_lin_kernel<128><<<grid, 256, 0, st>>>(ws_ptr<f32x4>(ws, wp.off_u), ws_ptr<float>(ws, wp.off_stat),
                                             ws_ptr<bf16x8>(ws, pl.off_sthi), ws_ptr<bf16x8>(ws, pl.off_stlo),
                                             ws_ptr<float>(ws, pl.off_z), ws_ptr<f32x4>(ws, wp.off_lin),
                                             ws_ptr<float>(ws, wp.off_e), pl.F, pl.N, wp.n_tb_q, pl.act_q, pl.P);
  return hipGetLastError();
}

}  // namespace ha
