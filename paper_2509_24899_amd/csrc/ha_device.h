// Device-side building blocks shared by the hybrid-attention kernels (gfx950 only).
//
// Every GEMM on the path runs on v_mfma_f32_32x32x16_bf16 (wave64).  Lane l = 32*g + r:
//   A operand (32 x 16): lane holds row r,  8 contraction slots (g, t), t = 0..7
//   B operand (16 x 32): lane holds col r,  the same 8 slots (g, t)
//   C / D    (32 x 32): register v of lane holds C[crow(v, g)][r],  crow = 8*(v/4) + 4*g + v%4
// The hardware pairs slot (g, t) of A with slot (g, t) of B, so which contraction index sits in a
// slot is the kernel's choice as long as both operands agree.  Two slot orders are used:
//   natural   slot (g, t) of k-step s  <->  index 16*s + 8*g + t            (operands read from
//             row-major memory as one 16-byte run)
//   chained   slot (g, t) of k-step s  <->  index 16*s + 8*(t/4) + 4*g + t%4   = crow(8*s + t, g)
//             (operand taken straight from the C registers 8*s .. 8*s+7 of a previous product)
// The chained order is what lets S^T = K Q^T feed O^T += V^T P^T, and the feature-map MLP feed
// the state contraction, without any trip through LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

static constexpr float kLog2e = 1.4426950408889634f;

static __device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of C register v for lane group g (also the chained slot order, see above).
static __device__ __forceinline__ constexpr int crow(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

// Kernels that gather bf16 weights straight from the caller's row-major tensors keep the hidden units of every 32-block
// in a permuted order: row rho of a layer-1 A fragment is weight row pi(rho), pi = swap of bits 2 and 3.  The C registers
// 8 s .. 8 s + 7 of layer 1, which feed layer 2 as its B operand, then hold hidden units 16 s + 8 g .. + 7 in order, so
// the matching A fragment piece of W2 is 16 contiguous bytes of a W2 row (no prepared, re-ordered copy of W2).
static __device__ __forceinline__ constexpr int perm_hidden(int rho) { return (rho & ~12) | ((rho & 4) << 1) | ((rho & 8) >> 1); }

// Combine a value with the lane that holds the other half of the same C column (lane ^ 32).
// v_permlane32_swap exchanges the upper half of one register with the lower half of another: called
// with the same value twice it hands every lane {its own value, the partner's} in some order.
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ float xhalf_max(float x) {
  const u32x2 p = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
}
static __device__ __forceinline__ float xhalf_sum(float x) {
  const u32x2 p = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}

static __device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 8 consecutive elements of a row in the io dtype -> 8 bf16 (fp32 is rounded to nearest even).
template <bool F32>
static __device__ __forceinline__ bf16x8 load8(const void *base, int64_t elem_off) {
  if constexpr (F32) {
    const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + elem_off);
    float4 a = p[0], b = p[1];
    f32x8 f = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    return __builtin_convertvector(f, bf16x8);
  } else {
    return *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(base) + elem_off);
  }
}

// Linear-token index -> token index: the tokens outside the softmax set in increasing order (R = 0: all).  With
// groups of G tokens, every R-th group being softmax tokens, linear token i lies in group-of-R-groups i / ((R - 1) G)
// and i + (that quotient + 1) G is its token index.  The quotient is exact for every int32 i: a double-precision
// reciprocal puts the estimate within one of the true floor, and one correction step settles it.
struct LinearMap {
  int d;        // (R - 1) G linear tokens per group of R G tokens, or a huge divisor when R == 0
  int g;        // G softmax tokens lead every group; 0 if R == 0
  double rcp;
  __device__ __forceinline__ LinearMap(int R, int G) : d(R == 0 ? 0x7fffffff : (R - 1) * G), g(R != 0 ? G : 0), rcp(1.0 / (double)d) {}
  __device__ __forceinline__ int token(int i) const {
    int q = (int)((double)i * rcp);
    int rem = i - q * d;
    q += (rem >= d) - (rem < 0);
    return i + (q + 1) * g;
  }
};

// Feature-map output stage on one C column held as NB row blocks of 16 registers (plus the same in
// lane ^ 32): positive activation over all channels, then channel c is raised to 1 + c / Dp.
//   act 0: softmax over the F = 32*NB channels;  1: exp;  2: relu.
// Dp is a multiple of 8 for every supported width, so the power of a channel depends only on its
// group of four registers (rows 32b + 8q .. + 7): the slice tests are wave-uniform.
template <int NB>
static __device__ __forceinline__ void feature_activation(f32x16 (&u)[NB], int g, int act, int P, int Dp) {
  (void)g;
  if (act == 0) {
    float mx = -INFINITY;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, u[b][v]);
    mx = xhalf_max(mx);
    const float off = -mx * kLog2e;
    float sum = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        u[b][v] = fast_exp2(__builtin_fmaf(u[b][v], kLog2e, off));
        sum += u[b][v];
      }
    sum = xhalf_sum(sum);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) u[b][v] *= inv;
  } else if (act == 1) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) u[b][v] = fast_exp2(u[b][v] * kLog2e);
  } else {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) u[b][v] = fmaxf(u[b][v], 0.f);
  }
  if (P > 1) {
    // slice p = c / Dp (0-based) gets p extra multiplications by the activation value
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int extra = ((32 * b + 8 * q) * P) / (32 * NB);   // = channel / Dp without a run-time division; wave-uniform
        if (extra > 0) {
          const float t0 = u[b][4 * q], t1 = u[b][4 * q + 1], t2 = u[b][4 * q + 2], t3 = u[b][4 * q + 3];
          for (int i = 0; i < extra; ++i) {
            u[b][4 * q] *= t0;
            u[b][4 * q + 1] *= t1;
            u[b][4 * q + 2] *= t2;
            u[b][4 * q + 3] *= t3;
          }
        }
      }
  }
}

// Two-layer feature-map MLP on one 32-token column block, all in registers.
//   xf[ks]  : B-operand fragments of the tokens (natural slot order over d)
//   w1f/w2f : A-operand fragments of the weights, w1 in natural order, w2 in chained order
// Layer 1 leaves relu(W1 x + b1) as hi + lo bf16 pairs in chained order: a peaky output softmax
// amplifies errors in u = W2 h + b2, so h is not allowed to lose its low mantissa bits.
// (WP: pointer to the weight fragments, global / generic `const bf16x8 *` or an LDS-qualified one)
// Fragment `idx` (64 lanes x 16 bytes) of an operand array: lane's piece.
//  - LDS-resident array: plain indexed read.
//  - array in global memory: read through a buffer descriptor, lane offset in one VGPR and the fragment offset in
//    a scalar register.  (With plain pointers the compiler precomputes one 64-bit per-lane address for every
//    fragment of a weight matrix, hoists them out of the loops and spills them.)  Reads past `bytes` return 0.
typedef const __attribute__((address_space(3))) bf16x8 *lds_frag_ptr;
struct GlobalFrags {
  const bf16x8 *base;
  int bytes;
};
static __device__ __forceinline__ GlobalFrags global_frags(const bf16x8 *base, int bytes) { return GlobalFrags{base, bytes}; }
// The descriptor is rebuilt at every use from a base address that is pinned to scalar registers: a descriptor
// the compiler parks in vector registers turns every read into a loop over its distinct values with a full
// wait behind it.  Word 3: raw 32-bit data format of gfx9-family buffers.
static __device__ __forceinline__ __amdgpu_buffer_rsrc_t frag_rsrc(const GlobalFrags &f) {
  const uint64_t p = reinterpret_cast<uint64_t>(f.base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(p));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(p >> 32));
  void *q = reinterpret_cast<void *>((static_cast<uint64_t>(hi) << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(q, 0, __builtin_amdgcn_readfirstlane(f.bytes), 0x00020000);
}
static __device__ __forceinline__ bf16x8 frag_at(lds_frag_ptr base, int idx, int lane) { return base[idx * 64 + lane]; }
static __device__ __forceinline__ bf16x8 frag_at(const GlobalFrags &f, int idx, int lane) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(frag_rsrc(f), lane * 16, idx * 1024, 0));
}
// n_chunks 1 KiB chunks global -> LDS with direct-to-LDS loads (no staging registers), dealt round-robin to the
// nw waves of the workgroup; wave index w must be wave-uniform.  The caller waits (vmcnt) and synchronises.
static __device__ __forceinline__ void dma_to_lds(const bf16x8 *gsrc, bf16x8 *ldst, int n_chunks, int w, int nw, int lane) {
  const unsigned lane_off16 = lane * 16;
  for (int ch = w; ch < n_chunks; ch += nw) {
    const unsigned l = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)(ldst + ch * 64));
    const bf16x8 *gp = gsrc + ch * 64;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(lane_off16), "s"(gp) : "memory");
  }
}

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;

// Transposing read: every 16 lanes form a group; lane j of a group receives, as its slot i, element j % 4 of what
// lane 4 i + j / 4 of the group addressed (4 consecutive 16-bit values).  With lane 4 i + a of a group pointing at
// columns c0 + 4 a .. + 3 of row T0 + i, lane j holds column c0 + j of rows T0 .. T0 + 3: four consecutive tokens of
// one column, i.e. half of a matrix-core operand fragment.
static __device__ __forceinline__ s16x4 ds_read_tr(const char *tile, int byte_off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + byte_off));
}
static __device__ __forceinline__ bf16x8 join(s16x4 a, s16x4 b) {
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Element e of the fragment arrays of one head's MLP weights (one thread per element):
//   w1f[h][hb][ks][lane][t] = W1[h][32hb + r][16ks + 8g + t]                       (natural order)
//   w2f[h][fb][hb][s][lane][t] = W2[h][32fb + r][32hb + crow(8s + t, g)]           (chained order)
template <bool F32>
static __device__ __forceinline__ void weight_prep_body(const void *__restrict__ w1, const void *__restrict__ w2,
                                                        __bf16 *__restrict__ w1f, __bf16 *__restrict__ w2f,
                                                        int D, int HD, int F, int h, int e) {
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


// A zero the compiler cannot see through.  Added to the scalar offset of fragment reads inside a loop whose
// fragments are the same in every iteration, it keeps those reads in the loop (hoisted, a whole operand matrix
// would sit in registers, i.e. in scratch).
static __device__ __forceinline__ int opaque_zero() {
  int z = 0;
  asm volatile("" : "+s"(z));
  return z;
}
static __device__ __forceinline__ bf16x8 frag_at(const GlobalFrags &f, int idx, int lane, int soff) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(frag_rsrc(f), lane * 16, idx * 1024 + soff, 0));
}

// BATCH: request all weight fragments of a block before its chain of matrix instructions starts, so the chain
// waits for LDS once instead of before every instruction; pays with one wave per SIMD, where nothing else
// hides the latency.  BP: pointer to the bias (global, or LDS-resident in the state pass).
template <int D, int HD, bool BATCH = false, typename WP, typename BP>
static __device__ __forceinline__ void feature_mlp_layer1(const bf16x8 (&xf)[D / 16], WP w1f,
                                                          BP b1, int lane, int g,
                                                          bf16x8 (&h_hi)[HD / 32][2], bf16x8 (&h_lo)[HD / 32][2]) {
  constexpr int KS = D / 16, HB = HD / 32;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    f32x16 h;
    if (b1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) h[v] = b1[32 * hb + crow(v, g)];
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) h[v] = 0.f;
    }
    if constexpr (BATCH) {
      // one wave per SIMD: all fragments of the block are requested before the chain starts, so the chain
      // waits for LDS once instead of before every instruction
      bf16x8 wf[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) wf[ks] = frag_at(w1f, hb * KS + ks, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) h = mfma32(wf[ks], xf[ks], h);
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) h = mfma32(frag_at(w1f, hb * KS + ks, lane), xf[ks], h);
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      f32x8 t, lo;
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = fmaxf(h[8 * s + i], 0.f);
      h_hi[hb][s] = __builtin_convertvector(t, bf16x8);
#pragma unroll
      for (int i = 0; i < 8; ++i) lo[i] = t[i] - static_cast<float>(h_hi[hb][s][i]);
      h_lo[hb][s] = __builtin_convertvector(lo, bf16x8);
    }
  }
}

// Layer 2: u[fb] = W2 h + b2 as C tiles (rows = channels, column = token).
template <int HD, int F, bool BATCH = false, typename WP, typename BP>
static __device__ __forceinline__ void feature_mlp_layer2(const bf16x8 (&h_hi)[HD / 32][2], const bf16x8 (&h_lo)[HD / 32][2],
                                                          WP w2f, BP b2,
                                                          int lane, int g, f32x16 (&u)[F / 32]) {
  constexpr int HB = HD / 32, FB = F / 32;
#pragma unroll
  for (int fb = 0; fb < FB; ++fb) {
    f32x16 acc;
    if (b2) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = b2[32 * fb + crow(v, g)];
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    }
    if constexpr (BATCH) {
      bf16x8 wf[HB][2];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int s = 0; s < 2; ++s) wf[hb][s] = frag_at(w2f, (fb * HB + hb) * 2 + s, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          acc = mfma32(wf[hb][s], h_lo[hb][s], acc);
          acc = mfma32(wf[hb][s], h_hi[hb][s], acc);
        }
    } else {
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const bf16x8 wf = frag_at(w2f, (fb * HB + hb) * 2 + s, lane);
          acc = mfma32(wf, h_lo[hb][s], acc);
          acc = mfma32(wf, h_hi[hb][s], acc);
        }
    }
    u[fb] = acc;
  }
}

// Layer 2 and the output stage fused, for wide maps (F > 128) where the fp32 pre-activations of all F
// channels of a token do not fit in registers next to everything else: every 32-channel tile is reduced
// to bf16 right after its chain of matrix instructions.  For the softmax activation this is an online
// softmax over the tiles: tile fb is exponentiated against the running maximum m_fb known so far and kept
// as bf16, and once all tiles are done it is rescaled by exp(m_fb - m) / sum, raised to its slice power and
// rounded again (two bf16 roundings instead of one; both are of the size the single rounding of the narrow
// path has).  phi[fb][s][i] is channel 32 fb + crow(8 s + i, g) of this lane's token: the B operand
// ("chained" order) of a product contracted over the channels.
template <int FB>
struct PhiState {
  float m_run = -INFINITY, sum = 0.f, mref[FB];
};

// Tiles FB0 .. FB1 - 1.  Fragment (fb, hb, s) of W2 is read at index (fb * HB + hb) * 2 + s - frag_bias, so a
// caller that stages W2 through LDS in pieces can hand in the piece that holds these tiles.
template <int HD, int F, int FB0, int FB1, bool BATCH, typename WP, typename BP>
static __device__ __forceinline__ void feature_layer2_phi_tiles(const bf16x8 (&h_hi)[HD / 32][2],
                                                                const bf16x8 (&h_lo)[HD / 32][2], WP w2f, int frag_bias,
                                                                BP b2, int lane, int g, int act, int P, int Dp,
                                                                PhiState<F / 32> &st, bf16x8 (&phi)[F / 32][2]) {
  constexpr int HB = HD / 32;
#pragma unroll
  for (int fb = FB0; fb < FB1; ++fb) {
    f32x16 acc;
    if (b2) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = b2[32 * fb + crow(v, g)];
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    }
    if constexpr (BATCH) {
      bf16x8 wf[HB][2];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int s = 0; s < 2; ++s) wf[hb][s] = frag_at(w2f, (fb * HB + hb) * 2 + s - frag_bias, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          acc = mfma32(wf[hb][s], h_lo[hb][s], acc);
          acc = mfma32(wf[hb][s], h_hi[hb][s], acc);
        }
    } else {
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const bf16x8 wf = frag_at(w2f, (fb * HB + hb) * 2 + s - frag_bias, lane);
          acc = mfma32(wf, h_lo[hb][s], acc);
          acc = mfma32(wf, h_hi[hb][s], acc);
        }
    }
    if (act == 0) {
      float t = acc[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) t = fmaxf(t, acc[v]);
      const float m_new = fmaxf(st.m_run, xhalf_max(t));
      st.sum *= fast_exp2((st.m_run - m_new) * kLog2e);          // exp2(-inf) = 0 on the first tile
      const float off = -m_new * kLog2e;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        acc[v] = fast_exp2(__builtin_fmaf(acc[v], kLog2e, off));
        st.sum += acc[v];
      }
      st.mref[fb] = m_new;
      st.m_run = m_new;
    } else if (act == 1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = fast_exp2(acc[v] * kLog2e);
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = fmaxf(acc[v], 0.f);
    }
    if (act != 0 && P > 1) {   // no normalisation to wait for: the slice power can be applied right away
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int extra = ((32 * fb + 8 * q) * P) / F;        // = channel / Dp; wave-uniform
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float t0 = acc[4 * q + j];
          for (int i = 0; i < extra; ++i) acc[4 * q + j] *= t0;
        }
      }
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      f32x8 t8;
#pragma unroll
      for (int i = 0; i < 8; ++i) t8[i] = acc[8 * s + i];
      phi[fb][s] = __builtin_convertvector(t8, bf16x8);
    }
  }
}

// After the last tile: the softmax normalisation and slice powers (nothing to do for the other activations).
template <int F>
static __device__ __forceinline__ void feature_phi_finish(const PhiState<F / 32> &st, int act, int P, int Dp,
                                                          bf16x8 (&phi)[F / 32][2]) {
  constexpr int FB = F / 32;
  if (act == 0) {
    const float inv = 1.0f / xhalf_sum(st.sum);
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) {
      const float factor = fast_exp2((st.mref[fb] - st.m_run) * kLog2e) * inv;
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        f32x8 t8;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float t0 = static_cast<float>(phi[fb][s][i]) * factor;
          const int extra = ((32 * fb + 8 * (2 * s + i / 4)) * P) / F;          // = channel / Dp; wave-uniform
          float t = t0;
          for (int k = 0; k < extra; ++k) t *= t0;
          t8[i] = t;
        }
        phi[fb][s] = __builtin_convertvector(t8, bf16x8);
      }
    }
  }
}

template <int HD, int F, bool BATCH, typename WP, typename BP>
static __device__ __forceinline__ void feature_layer2_phi(const bf16x8 (&h_hi)[HD / 32][2], const bf16x8 (&h_lo)[HD / 32][2],
                                                          WP w2f, BP b2, int lane, int g, int act, int P, int Dp,
                                                          bf16x8 (&phi)[F / 32][2]) {
  PhiState<F / 32> st;
  feature_layer2_phi_tiles<HD, F, 0, F / 32, BATCH>(h_hi, h_lo, w2f, 0, b2, lane, g, act, P, Dp, st, phi);
  feature_phi_finish<F>(st, act, P, Dp, phi);
}

template <int D, int HD, int F, typename WP>
static __device__ __forceinline__ void feature_mlp(const bf16x8 (&xf)[D / 16], WP w1f,
                                                   WP w2f, const float *b1,
                                                   const float *b2, int lane, int g,
                                                   f32x16 (&u)[F / 32]) {
  bf16x8 h_hi[HD / 32][2], h_lo[HD / 32][2];
  feature_mlp_layer1<D, HD>(xf, w1f, b1, lane, g, h_hi, h_lo);
  feature_mlp_layer2<HD, F>(h_hi, h_lo, w2f, b2, lane, g, u);
}

}  // namespace ha
