// The feature map phi of Sec. 3.2 for the widths 128 -> 128 -> 128 on one 32-token column block, as the hand-placed
// software pipeline the state pass and the gradient pass share.  gfx950 only.
//   * Layer 1 runs two row blocks at a time (two independent accumulator chains, their matrix instructions
//     alternate); the fragments of the second pair arrive four k-steps ahead of their use, and its matrix
//     instructions carry the ReLU / hi + lo conversion of the first pair.
//   * Layer 2 runs two output tiles at a time in steps of one hidden block; the fragments of the next step are
//     requested behind the step's first matrix instruction.  Under the steps: first the conversion of layer-1 blocks
//     2, 3, later (softmax output) the exponentials of the finished pair of tiles against their own maximum; the
//     second pair is exponentiated against the overall maximum, one factor per pair at the end.
#pragma once
#include "ha_device.h"

namespace ha {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
static __device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  const f32x2 t = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2));
}
// Nothing moves across: the instruction order between two fences is the compiler's, the order of the fenced groups
// is the source's.  The kernel below places its matrix instructions, LDS reads and vector work by hand with it.
#define HA_FENCE() __builtin_amdgcn_sched_barrier(0)


// xf: the B-operand fragments of the 32 token rows (natural slot order over d); w1f / w2f: A-operand fragments of the
// weights in LDS (W1 natural order, W2 in the order of the C registers of layer 1); b1, b2: the biases in LDS.
// Out: h_hi / h_lo = relu(W1 x + b1) as hi + lo bf16 pairs in chained order, u = the positive output activation of
// W2 h + b2 (before the slice powers).  ACT0: the activation is the softmax over the channels (scheduled by hand);
// `act` picks exp (1) or ReLU otherwise.  between_layers() is called once layer 1 no longer needs xf.
// LEAN: the fragments of the first pair of layer-1 blocks arrive four k-steps ahead of their use as well (32 registers
// less, for a caller with less room).
template <bool ACT0, bool LEAN = false, typename MID>
static __device__ __forceinline__ void mlp128_pipelined(const bf16x8 (&xf)[8], lds_frag_ptr w1f, lds_frag_ptr w2f, const float *b1,
                                                        const float *b2, int lane, int g, int act, u32x4 (&h_hi)[4][2],
                                                        u32x4 (&h_lo)[4][2], f32x16 (&u)[4], MID between_layers) {
  constexpr int KS = 8, HB = 4, FB = 4;
  // a chain's accumulator starts as the bias of its 32 channels: four 16-byte LDS reads (registers 4 v .. 4 v + 3 are
  // four consecutive channels), no vector instruction
  auto bias_tile = [&](const float *b, int blk) {
    const f32x4 *src = reinterpret_cast<const f32x4 *>(b + 32 * blk + 4 * g);
    const f32x8 lo = __builtin_shufflevector(src[0], src[2], 0, 1, 2, 3, 4, 5, 6, 7);
    const f32x8 hi = __builtin_shufflevector(src[4], src[6], 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
  };
  // registers x, x + 1 of a finished layer-1 tile -> ReLU -> hi + lo (8 vector instructions)
  auto conv2 = [&](const f32x16 &hh, int hb, int x) {
    const float a = fmaxf(hh[x], 0.f), b = fmaxf(hh[x + 1], 0.f);
    const unsigned hi = pack_bf16(a, b);
    h_hi[hb][x >> 3][(x & 7) >> 1] = hi;
    h_lo[hb][x >> 3][(x & 7) >> 1] = pack_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
  };
  auto hop = [&](const u32x4 &t) { return __builtin_bit_cast(bf16x8, t); };
  {
    // ---------------- layer 1: two row blocks at a time (two independent chains, alternating); the fragments of
    // the second pair arrive four k-steps ahead of their use
    f32x16 ha0, ha1, ha2, ha3;
    bf16x8 wA[2][LEAN ? KS / 2 : KS], wB[2][KS / 2];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int ks = 0; ks < (LEAN ? KS / 2 : KS); ++ks) wA[e][ks] = frag_at(w1f, e * KS + ks, lane);
    ha0 = bias_tile(b1, 0);
    ha1 = bias_tile(b1, 1);
    ha2 = bias_tile(b1, 2);
    ha3 = bias_tile(b1, 3);
    HA_FENCE();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {              // blocks 0, 1
      ha0 = mfma32(wA[0][LEAN ? ks % (KS / 2) : ks], xf[ks], ha0);
      if (LEAN && ks < KS / 2) wA[0][ks] = frag_at(w1f, 0 * KS + ks + KS / 2, lane);
      if (ks >= KS / 2) wB[0][ks - KS / 2] = frag_at(w1f, 2 * KS + ks - KS / 2, lane);
      HA_FENCE();
      ha1 = mfma32(wA[1][LEAN ? ks % (KS / 2) : ks], xf[ks], ha1);
      if (LEAN && ks < KS / 2) wA[1][ks] = frag_at(w1f, 1 * KS + ks + KS / 2, lane);
      if (ks >= KS / 2) wB[1][ks - KS / 2] = frag_at(w1f, 3 * KS + ks - KS / 2, lane);
      HA_FENCE();
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {              // blocks 2, 3 under the conversion of blocks 0, 1
      ha2 = mfma32(wB[0][ks % (KS / 2)], xf[ks], ha2);
      if (ks < KS / 2) wB[0][ks] = frag_at(w1f, 2 * KS + ks + KS / 2, lane);
      conv2(ha0, 0, 2 * ks);
      ha3 = mfma32(wB[1][ks % (KS / 2)], xf[ks], ha3);
      if (ks < KS / 2) wB[1][ks] = frag_at(w1f, 3 * KS + ks + KS / 2, lane);
      conv2(ha1, 1, 2 * ks);
    }
    // one matrix instruction, then one conversion's worth of vector instructions, sixteen times; the accumulators
    // are tied to the end of this stretch so that the matrix instructions cannot drift out of it
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
    }
    asm volatile("" : "+v"(ha2), "+v"(ha3));
    HA_FENCE();
    between_layers();                              // (the caller requests the rows of its next tile here)
    HA_FENCE();

    // ---------------- layer 2: u = W2 h + b2, two 32-channel tiles at a time, one hidden block (8 matrix
    // instructions, 4 fragments) per step; the fragments of the next step are requested behind the step's first
    // matrix instruction.  Under the steps: first the conversion of layer-1 blocks 2, 3, later the softmax
    // exponentials of the finished pair of tiles.
    bf16x8 wa[2][2], wb[2][2];
    auto w2_frags = [&](int fp, int hb, bf16x8 (&dst)[2][2]) {
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int s = 0; s < 2; ++s) dst[e][s] = frag_at(w2f, ((fp + e) * HB + hb) * 2 + s, lane);
    };
    w2_frags(0, 0, wa);
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) u[fb] = bias_tile(b2, fb);
    float m0 = 0.f, off0 = 0.f, sum0 = 0.f;
    HA_FENCE();
#pragma unroll
    for (int fp = 0; fp < FB; fp += 2) {
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        bf16x8 (&cur)[2][2] = (hb & 1) ? wb : wa;
        bf16x8 (&nxt)[2][2] = (hb & 1) ? wa : wb;
#pragma unroll
        for (int slot = 0; slot < 8; ++slot) {
          const int e = slot & 1, hi = (slot >> 1) & 1, s = slot >> 2;
          u[fp + e] = mfma32(cur[e][s], hop(hi ? h_hi[hb][s] : h_lo[hb][s]), u[fp + e]);
          if (slot == 0) {
            if (hb + 1 < HB) w2_frags(fp, hb + 1, nxt);
            else if (fp + 2 < FB) w2_frags(fp + 2, 0, nxt);
          }
          const int n = hb * 8 + slot;             // 0 .. 31 within the pair
          if (fp == 0) {
            if (n < 8) conv2(ha2, 2, 2 * n);       // needed from step 2 on
            else if (n < 16) conv2(ha3, 3, 2 * (n - 8));
          } else if constexpr (ACT0) {
            // softmax of tiles 0, 1: their maximum in the first two slots, then one exponential per slot
            if (n == 0) {
              float t = fmaxf(u[0][0], u[0][1]);
#pragma unroll
              for (int x = 2; x < 16; x += 2) t = __builtin_fmaxf(__builtin_fmaxf(t, u[0][x]), u[0][x + 1]);
              m0 = t;
            } else if (n == 1) {
              float t = m0;
#pragma unroll
              for (int x = 0; x < 16; x += 2) t = __builtin_fmaxf(__builtin_fmaxf(t, u[1][x]), u[1][x + 1]);
              m0 = xhalf_max(t);
              off0 = -m0 * kLog2e;
            } else {
              auto ex = [&](int i) {
                u[i >> 4][i & 15] = fast_exp2(__builtin_fmaf(u[i >> 4][i & 15], kLog2e, off0));
                sum0 += u[i >> 4][i & 15];
              };
              ex(n - 2);
              if (n >= 30) ex(n);                  // 30 slots for 32 values: the last two slots take two each
            }
          }
          HA_FENCE();
        }
      }
    }
    if constexpr (ACT0) {
      // tiles 2, 3 against the overall maximum, which is known now
      float t = fmaxf(u[2][0], u[2][1]);
#pragma unroll
      for (int x = 2; x < 16; x += 2) t = __builtin_fmaxf(__builtin_fmaxf(t, u[2][x]), u[2][x + 1]);
#pragma unroll
      for (int x = 0; x < 16; x += 2) t = __builtin_fmaxf(__builtin_fmaxf(t, u[3][x]), u[3][x + 1]);
      const float m = fmaxf(m0, xhalf_max(t));
      const float off = -m * kLog2e;
      float sum1 = 0.f;
#pragma unroll
      for (int fb = 2; fb < 4; ++fb)
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          u[fb][x] = fast_exp2(__builtin_fmaf(u[fb][x], kLog2e, off));
          sum1 += u[fb][x];
        }
      const float carry = fast_exp2((m0 - m) * kLog2e);        // tiles 0, 1 were exponentiated against m0
      const float inv = 1.0f / xhalf_sum(sum0 * carry + sum1);
      const float f0 = carry * inv;
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        u[0][x] *= f0;
        u[1][x] *= f0;
        u[2][x] *= inv;
        u[3][x] *= inv;
      }
    } else if (act == 1) {
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int x = 0; x < 16; ++x) u[fb][x] = fast_exp2(u[fb][x] * kLog2e);
    } else {
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int x = 0; x < 16; ++x) u[fb][x] = fmaxf(u[fb][x], 0.f);
    }
  }
}

}  // namespace ha
