// HIP kernels of the hybrid-attention forward (Attention Surgery, Sec. 3.2, Eq. "hybrid"), gfx950.
//
//   weight_prep_kernel   MLP weights -> bf16 A-operand fragments (once per call, tiny)
//   compact_kernel       softmax tokens T_S (every R-th token, Sec. 3.2): K_S and V_S gathered into
//                        matrix-core fragment order, zero padded to whole key tiles
//   state_kernel         linear tokens T_L: phi_k(k_j), then partial S = sum phi_k(k_j)^T v_j and
//                        z = sum phi_k(k_j) per chunk of tokens (Sec. 3.1: the two cached sums)
//   state_reduce_kernel  fixed-order sum of the partials -> S, z (fp32) and S^T as hi/lo bf16 fragments
//   query_kernel         per 32-query column block: flash-style loop over K_S/V_S with online
//                        maximum c_i, then phi_q(q_i), phi_q(q_i).S, phi_q(q_i).z and the merge
//                        (a_i + n_i) / (l_i + e_i) of Eq. "hybrid"
//
// All products are computed transposed (keys x queries, channels x tokens) so that one lane owns one
// query / token column: row maxima and sums are in-lane plus one exchange with lane ^ 32.
#include "ha_device.h"
#include "ha_plan.h"

namespace ha {

// ------------------------------------------------------------------------------------------------
// weight_prep_kernel: grid (ceil(max(HD*D, F*HD) / 256), H)
//   w1f[h][hb][ks][lane][t] = W1[h][32hb + r][16ks + 8g + t]                       (natural order)
//   w2f[h][fb][hb][s][lane][t] = W2[h][32fb + r][32hb + crow(8s + t, g)]           (chained order)
template <bool F32>
__global__ __launch_bounds__(256) void weight_prep_kernel(const void *__restrict__ w1, const void *__restrict__ w2,
                                                          __bf16 *__restrict__ w1f, __bf16 *__restrict__ w2f,
                                                          int D, int HD, int F) {
  const int h = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int t = e & 7, lane = (e >> 3) & 63, rest = e >> 9;
  const int r = lane & 31, g = lane >> 5;
  auto ld = [](const void *p, int64_t i) -> float {
    if constexpr (F32) return static_cast<const float *>(p)[i];
    else return static_cast<float>(static_cast<const __bf16 *>(p)[i]);
  };
  if (e < HD * D) {
    const int KS = D / 16;
    const int ks = rest % KS, hb = rest / KS;
    w1f[(int64_t)h * HD * D + e] = static_cast<__bf16>(ld(w1, ((int64_t)h * HD + 32 * hb + r) * D + 16 * ks + 8 * g + t));
  }
  if (e < F * HD) {
    const int HB = HD / 32;
    const int s = rest & 1, hb = (rest >> 1) % HB, fb = (rest >> 1) / HB;
    w2f[(int64_t)h * F * HD + e] =
        static_cast<__bf16>(ld(w2, ((int64_t)h * F + 32 * fb + r) * HD + 32 * hb + crow(8 * s + t, g)));
  }
}

// ------------------------------------------------------------------------------------------------
// compact_kernel: grid (n_kblocks, B*H); one workgroup builds one 32-key block of both fragment arrays.
//   ks_frag[bh][kb][ks][lane]          = K[token(32kb + r)][16ks + 8g .. +7]
//   vs_frag[bh][kb][rb][s][lane][t]    = V[token(32kb + crow(8s + t, g))][32rb + r]
// token(key) = key * R; keys >= NS are zero padding.
template <int D, bool F32>
__global__ __launch_bounds__(256) void compact_kernel(const void *__restrict__ k, const void *__restrict__ v,
                                                      bf16x8 *__restrict__ ks_frag, bf16x8 *__restrict__ vs_frag,
                                                      int H, int NS, int R, int n_kblocks, int64_t sb, int64_t sh,
                                                      int64_t sn) {
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
      const int64_t off = base + (int64_t)key * R * sn + c8 * 8;
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
template <int D, int HD, int F, bool F32>
__global__ __launch_bounds__(256) void state_kernel(const void *__restrict__ k, const void *__restrict__ v,
                                                    const bf16x8 *__restrict__ w1f_all, const bf16x8 *__restrict__ w2f_all,
                                                    const float *__restrict__ b1_all, const float *__restrict__ b2_all,
                                                    float *__restrict__ part, int H, int NL, int R, int CH, int P,
                                                    int act, int64_t sb, int64_t sh, int64_t sn) {
  constexpr int TOK = 128, PITCH = TOK + 8;
  constexpr int KS = D / 16, FB = F / 32, NCB = D / 32 + 1, NT = FB * NCB, TPW = (NT + 3) / 4;
  __shared__ __align__(16) __bf16 ft[F][PITCH];
  __shared__ __align__(16) __bf16 vt[D][PITCH];
  const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % H;
  const int64_t base = (int64_t)(bh / H) * sb + (int64_t)h * sh;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const bf16x8 *w1f = w1f_all + (int64_t)h * (HD * D / 8);
  const bf16x8 *w2f = w2f_all + (int64_t)h * (F * HD / 8);
  const float *b1 = b1_all ? b1_all + (int64_t)h * HD : nullptr;
  const float *b2 = b2_all ? b2_all + (int64_t)h * F : nullptr;
  const int Dp = F / P;

  f32x16 acc[TPW];
#pragma unroll
  for (int i = 0; i < TPW; ++i)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[i][x] = 0.f;

  const int lt_begin = chunk * CH;
  const int lt_end = min(lt_begin + CH, NL);
  for (int t0 = lt_begin; t0 < lt_end; t0 += TOK) {
    // phi_k on this wave's 32 tokens
    {
      const int lt = t0 + w * 32 + r;
      const bool valid = lt < NL;
      const int tok = linear_to_token(valid ? lt : NL - 1, R);
      bf16x8 xf[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) xf[ks] = load8<F32>(k, base + (int64_t)tok * sn + 16 * ks + 8 * g);
      f32x16 u[FB];
      feature_mlp<D, HD, F>(xf, w1f, w2f, b1, b2, lane, g, u);
      feature_activation<FB>(u, g, act, P, Dp);
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int x = 0; x < 16; ++x)
          ft[32 * fb + crow(x, g)][w * 32 + r] = static_cast<__bf16>(valid ? u[fb][x] : 0.f);
    }
    // V^T of the tile's 128 tokens
    for (int c = tid; c < TOK * (D / 8); c += 256) {
      const int trow = c / (D / 8), c8 = c % (D / 8);
      const int lt = min(t0 + trow, NL - 1);
      const bf16x8 vv = load8<F32>(v, base + (int64_t)linear_to_token(lt, R) * sn + c8 * 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) vt[c8 * 8 + i][trow] = vv[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
      const int ti = w + 4 * i;
      if (ti < NT) {
        const int fb = ti / NCB, cb = ti % NCB;
#pragma unroll
        for (int ks = 0; ks < TOK / 16; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&ft[32 * fb + r][16 * ks + 8 * g]);
          bf16x8 b;
          if (cb < D / 32) {
            b = *reinterpret_cast<const bf16x8 *>(&vt[32 * cb + r][16 * ks + 8 * g]);
          } else {
            const __bf16 one = static_cast<__bf16>(r == 0 ? 1.0f : 0.0f);   // the "1" column that yields z
            b = bf16x8{one, one, one, one, one, one, one, one};
          }
          acc[i] = mfma32(a, b, acc[i]);
        }
      }
    }
    __syncthreads();
  }
  float *dst = part + ((int64_t)bh * gridDim.x + chunk) * NT * 1024;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int ti = w + 4 * i;
    if (ti < NT) {
#pragma unroll
      for (int x = 0; x < 16; ++x) dst[ti * 1024 + x * 64 + lane] = acc[i][x];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// state_reduce_kernel: grid (NT*1024/256, B*H).  Sums the chunk partials in chunk order (bitwise
// reproducible), writes S [F][D] and z [F] in fp32, and S^T split into hi + lo bf16 in the
// A-operand order of the query kernel:  st[bh][rb][fb][s][lane][t] = S[32fb + crow(8s + t, g)][32rb + r].
__global__ __launch_bounds__(256) void state_reduce_kernel(const float *__restrict__ part, float *__restrict__ S,
                                                           float *__restrict__ z, __bf16 *__restrict__ st_hi,
                                                           __bf16 *__restrict__ st_lo, int D, int F, int n_chunks) {
  const int NCB = D / 32 + 1, FB = F / 32, NT = FB * NCB;
  const int bh = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= NT * 1024) return;
  const int ti = e >> 10, x = (e >> 6) & 15, lane = e & 63, r = lane & 31, g = lane >> 5;
  float sum = 0.f;
  for (int c = 0; c < n_chunks; ++c) sum += part[((int64_t)bh * n_chunks + c) * NT * 1024 + e];
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

// ------------------------------------------------------------------------------------------------
// query_kernel: 4 waves; wave w owns QB column blocks of 32 queries.  Workgroups are numbered so that
// consecutive ids on one XCD (id % 8) walk the query tiles of one (batch, head) together and share its
// K_S / V_S in that XCD's L2.
struct QueryArgs {
  const void *q;
  void *out;
  const bf16x8 *ks_frag, *vs_frag;       // [B*H][n_kblocks][D*4]
  const bf16x8 *w1f, *w2f;               // phi_q fragments, per head
  const float *b1, *b2;                 // phi_q biases, per head (may be null)
  const bf16x8 *st_hi, *st_lo;           // [B*H][D/32][F/32][2][64]
  const float *z;                       // [B*H][F]
  int H, N, NS, n_qtiles, n_ktiles, n_kblocks, total_wg;
  int has_linear, P, act;
  int64_t sb, sh, sn;
  float scale_log2e;
};

template <int D, int HD, int F, int QB, int KT, bool F32>
__global__ __launch_bounds__(256, (QB == 1 ? 2 : 1)) void query_kernel(QueryArgs a) {
  constexpr int KS = D / 16, RB = D / 32, FB = F / 32;
  constexpr int KBT = KT / 32;          // 32-key blocks per LDS tile
  constexpr int FRAG = D * 4;           // bf16x8 per key block, same for K and V
  constexpr int NLD = KBT * FRAG / 256; // bf16x8 per thread per tile per tensor
  constexpr int QT = 128 * QB;
  __shared__ bf16x8 lds_k[2][KBT * FRAG];
  __shared__ bf16x8 lds_v[2][KBT * FRAG];

  // XCD-aware numbering: hardware deals workgroup ids round-robin over the 8 XCDs.
  const int per_xcd = (a.total_wg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= a.total_wg) return;
  const int bh = logical / a.n_qtiles, qtile = logical % a.n_qtiles;
  const int h = bh % a.H;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int q0 = qtile * QT + w * (32 * QB);

  // Q^T as B-operand fragments, natural order over d
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qi = min(q0 + 32 * qb + r, a.N - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = load8<F32>(a.q, base + (int64_t)qi * a.sn + 16 * ks + 8 * g);
  }

  f32x16 o[RB][QB];
  float m[QB], lsum[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m[qb] = -INFINITY;
    lsum[qb] = 0.f;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int x = 0; x < 16; ++x) o[rb][qb][x] = 0.f;
  }

  if (a.n_ktiles > 0) {
    const bf16x8 *ksrc = a.ks_frag + (int64_t)bh * a.n_kblocks * FRAG;
    const bf16x8 *vsrc = a.vs_frag + (int64_t)bh * a.n_kblocks * FRAG;
    bf16x8 stk[NLD], stv[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      stk[i] = ksrc[i * 256 + tid];
      stv[i] = vsrc[i * 256 + tid];
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      lds_k[0][i * 256 + tid] = stk[i];
      lds_v[0][i * 256 + tid] = stv[i];
    }
    __syncthreads();
    const float c = a.scale_log2e;
    for (int t = 0; t < a.n_ktiles; ++t) {
      const int buf = t & 1;
      const bool more = t + 1 < a.n_ktiles;
      if (more) {
        const int64_t off = (int64_t)(t + 1) * KBT * FRAG;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          stk[i] = ksrc[off + i * 256 + tid];
          stv[i] = vsrc[off + i * 256 + tid];
        }
      }
      const bool tail = (t == a.n_ktiles - 1) && (a.NS % KT != 0);
#pragma unroll
      for (int step = 0; step < KBT / 2; ++step) {
        const int key0 = t * KT + step * 64;
        if (key0 < a.NS) {
          // S^T = K Q^T for 64 keys x (32*QB) queries
          f32x16 s[2][QB];
#pragma unroll
          for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
              for (int x = 0; x < 16; ++x) s[kb][qb][x] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
              const bf16x8 kf = lds_k[buf][(step * 2 + kb) * FRAG + ks * 64 + lane];
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) s[kb][qb] = mfma32(kf, qf[qb][ks], s[kb][qb]);
            }
          }
          if (tail) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int x = 0; x < 16; ++x) {
                const bool dead = key0 + 32 * kb + crow(x, g) >= a.NS;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) s[kb][qb][x] = dead ? -INFINITY : s[kb][qb][x];
              }
          }
          // online softmax per query column; c_i stays the exact running maximum
          bf16x8 pb[2][2][QB];
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int x = 0; x < 16; ++x) mx = fmaxf(mx, s[kb][qb][x]);
            mx = xhalf_max(mx);
            const float m_new = fmaxf(m[qb], mx);
            if (__any(m_new > m[qb])) {
              const float alpha = fast_exp2((m[qb] - m_new) * c);
              lsum[qb] *= alpha;
#pragma unroll
              for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int x = 0; x < 16; ++x) o[rb][qb][x] *= alpha;
              m[qb] = m_new;
            }
            const float mc = m[qb] * c;
            float ps = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int sp = 0; sp < 2; ++sp) {
                f32x8 p8;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                  p8[i] = fast_exp2(__builtin_fmaf(s[kb][qb][8 * sp + i], c, -mc));
                  ps += p8[i];
                }
                pb[kb][sp][qb] = __builtin_convertvector(p8, bf16x8);
              }
            lsum[qb] += ps;
          }
          // O^T += V^T P^T
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int sp = 0; sp < 2; ++sp)
#pragma unroll
              for (int rb = 0; rb < RB; ++rb) {
                const bf16x8 vf = lds_v[buf][(step * 2 + kb) * FRAG + (rb * 2 + sp) * 64 + lane];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) o[rb][qb] = mfma32(vf, pb[kb][sp][qb], o[rb][qb]);
              }
        }
      }
      if (more) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          lds_k[buf ^ 1][i * 256 + tid] = stk[i];
          lds_v[buf ^ 1][i * 256 + tid] = stv[i];
        }
      }
      __syncthreads();
    }
  }

  // epilogue per query column block: linear part and merge
  const bf16x8 *w1f = a.w1f + (int64_t)h * (HD * D / 8);
  const bf16x8 *w2f = a.w2f + (int64_t)h * (F * HD / 8);
  const float *b1 = a.b1 ? a.b1 + (int64_t)h * HD : nullptr;
  const float *b2 = a.b2 ? a.b2 + (int64_t)h * F : nullptr;
  const int Dp = F / a.P;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    float den = xhalf_sum(lsum[qb]);
    if (a.has_linear) {
      f32x16 u[FB];
      feature_mlp<D, HD, F>(qf[qb], w1f, w2f, b1, b2, lane, g, u);
      feature_activation<FB>(u, g, a.act, a.P, Dp);
      bf16x8 gb[FB][2];
      float e = 0.f;
      const float *zz = a.z + (int64_t)bh * F;
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
          f32x8 t8;
#pragma unroll
          for (int i = 0; i < 8; ++i) t8[i] = u[fb][8 * sp + i];
          gb[fb][sp] = __builtin_convertvector(t8, bf16x8);
#pragma unroll
          for (int i = 0; i < 8; ++i) e += static_cast<float>(gb[fb][sp][i]) * zz[32 * fb + crow(8 * sp + i, g)];
        }
      den += xhalf_sum(e);
      const bf16x8 *sth = a.st_hi + (int64_t)bh * (RB * FB * 2 * 64);
      const bf16x8 *stl = a.st_lo + (int64_t)bh * (RB * FB * 2 * 64);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        f32x16 n;
#pragma unroll
        for (int x = 0; x < 16; ++x) n[x] = 0.f;
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
          for (int sp = 0; sp < 2; ++sp) {
            const int idx = ((rb * FB + fb) * 2 + sp) * 64 + lane;
            n = mfma32(stl[idx], gb[fb][sp], n);
            n = mfma32(sth[idx], gb[fb][sp], n);
          }
#pragma unroll
        for (int x = 0; x < 16; ++x) o[rb][qb][x] += n[x];
      }
    }
    const float inv = 1.0f / den;
    const int qi = q0 + 32 * qb + r;
    if (qi < a.N) {
      const int64_t ooff = base + (int64_t)qi * a.sn;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int x4 = 0; x4 < 4; ++x4) {
          const int dcol = 32 * rb + 8 * x4 + 4 * g;
          f32x4 y = {o[rb][qb][4 * x4] * inv, o[rb][qb][4 * x4 + 1] * inv, o[rb][qb][4 * x4 + 2] * inv,
                     o[rb][qb][4 * x4 + 3] * inv};
          if constexpr (F32) {
            *reinterpret_cast<f32x4 *>(static_cast<float *>(a.out) + ooff + dcol) = y;
          } else {
            *reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(a.out) + ooff + dcol) = __builtin_convertvector(y, bf16x4);
          }
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
  compact_kernel<DD, FF><<<grid, 256, 0, st>>>(k, v, ksf, vsf, pl.H, pl.NS, pl.R, pl.n_kblocks, pl.sb, pl.sh, pl.sn)
  if (pl.D == 64) { if (pl.f32) HA_COMPACT(64, true); else HA_COMPACT(64, false); }
  else { if (pl.f32) HA_COMPACT(128, true); else HA_COMPACT(128, false); }
#undef HA_COMPACT
  return hipGetLastError();
}

hipError_t launch_state(const Plan &pl, const void *k, const void *v, const ha_feature_map &fm, void *ws,
                        hipStream_t st) {
  dim3 grid(pl.n_chunks, pl.B * pl.H);
  const bf16x8 *w1f = ws_ptr<bf16x8>(ws, pl.off_w1k), *w2f = ws_ptr<bf16x8>(ws, pl.off_w2k);
  float *part = ws_ptr<float>(ws, pl.off_part);
#define HA_STATE(DD, HH, FF, F32) \
  state_kernel<DD, HH, FF, F32><<<grid, 256, 0, st>>>(k, v, w1f, w2f, fm.b1, fm.b2, part, pl.H, pl.NL, pl.R, pl.CH, \
                                                     pl.P, pl.act_k, pl.sb, pl.sh, pl.sn)
  if (pl.D == 64) { if (pl.f32) HA_STATE(64, 64, 64, true); else HA_STATE(64, 64, 64, false); }
  else if (pl.HD == 128) { if (pl.f32) HA_STATE(128, 128, 128, true); else HA_STATE(128, 128, 128, false); }
  else { if (pl.f32) HA_STATE(128, 256, 256, true); else HA_STATE(128, 256, 256, false); }
#undef HA_STATE
  return hipGetLastError();
}

hipError_t launch_state_reduce(const Plan &pl, void *ws, hipStream_t st) {
  dim3 grid(pl.n_state_tiles * 1024 / 256, pl.B * pl.H);
  state_reduce_kernel<<<grid, 256, 0, st>>>(ws_ptr<float>(ws, pl.off_part), ws_ptr<float>(ws, pl.off_S),
                                            ws_ptr<float>(ws, pl.off_z), ws_ptr<__bf16>(ws, pl.off_sthi),
                                            ws_ptr<__bf16>(ws, pl.off_stlo), pl.D, pl.F, pl.n_chunks);
  return hipGetLastError();
}

hipError_t launch_query(const Plan &pl, const void *q, const ha_feature_map *phi_q, void *out, void *ws,
                        hipStream_t st) {
  QueryArgs a;
  a.q = q;
  a.out = out;
  a.ks_frag = ws_ptr<bf16x8>(ws, pl.off_ks);
  a.vs_frag = ws_ptr<bf16x8>(ws, pl.off_vs);
  a.w1f = ws_ptr<bf16x8>(ws, pl.off_w1q);
  a.w2f = ws_ptr<bf16x8>(ws, pl.off_w2q);
  a.b1 = phi_q ? phi_q->b1 : nullptr;
  a.b2 = phi_q ? phi_q->b2 : nullptr;
  a.st_hi = ws_ptr<bf16x8>(ws, pl.off_sthi);
  a.st_lo = ws_ptr<bf16x8>(ws, pl.off_stlo);
  a.z = ws_ptr<float>(ws, pl.off_z);
  a.H = pl.H; a.N = pl.N; a.NS = pl.NS;
  a.n_qtiles = pl.n_qtiles; a.n_ktiles = pl.n_ktiles; a.n_kblocks = pl.n_kblocks;
  a.total_wg = pl.n_qtiles * pl.B * pl.H;
  a.has_linear = pl.NL > 0; a.P = pl.P; a.act = pl.act_q;
  a.sb = pl.sb; a.sh = pl.sh; a.sn = pl.sn;
  a.scale_log2e = pl.scale * kLog2e;
  dim3 grid(((a.total_wg + 7) / 8) * 8);
#define HA_QUERY(DD, HH, FF, F32) \
  do { \
    if (pl.QB == 1) query_kernel<DD, HH, FF, 1, 64, F32><<<grid, 256, 0, st>>>(a); \
    else query_kernel<DD, HH, FF, 2, 128, F32><<<grid, 256, 0, st>>>(a); \
  } while (0)
  if (pl.D == 64) { if (pl.f32) HA_QUERY(64, 64, 64, true); else HA_QUERY(64, 64, 64, false); }
  else if (pl.HD == 128) { if (pl.f32) HA_QUERY(128, 128, 128, true); else HA_QUERY(128, 128, 128, false); }
  else { if (pl.f32) HA_QUERY(128, 256, 256, true); else HA_QUERY(128, 256, 256, false); }
#undef HA_QUERY
  return hipGetLastError();
}

}  // namespace ha
