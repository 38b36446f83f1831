// Query-side kernels of the hybrid-attention forward (Attention Surgery, Sec. 3.2, Eq. "hybrid"), gfx950.
#include <type_traits>

#include "ha_device.h"
#include "ha_plan.h"

namespace ha {

template <typename T>
static inline T *ws_ptr(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }

// ------------------------------------------------------------------------------------------------
// Arguments of the query kernel.  Workgroups are numbered so that consecutive ids on one XCD (id % 8) walk the
// query tiles of one (batch, head) together and share its K_S / V_S in that XCD's L2.
struct QueryArgs {
  const void *q;
  void *out;
  const bf16x8 *ks_frag, *vs_frag;       // [B*H][n_kblocks][D*4]
  const bf16x8 *w1f, *w2f;               // phi_q fragments, per head
  const float *b1, *b2;                 // phi_q biases, per head (may be null)
  const bf16x8 *st_hi, *st_lo;           // [B*H][D/32][F/32][2][64]
  const float *z;                       // [B*H][F]
  float *row_den;                       // optional [B*H][N]: the denominator l_i + phi_q(q_i).z of every row
  // maps too wide for the fused epilogue: n_i = phi_q(q_i) S and e_i = phi_q(q_i).z arrive precomputed
  const f32x4 *lin;                     // [B*H][n_tb][D/32][4][64]: fp32 register image of n^T per 32-query block, or null
  const float *lin_e;                   // [B*H][N]
  int n_tb;
  int H, N, NS, n_qtiles, n_ktiles, n_kblocks, total_wg;
  int CC, n_cc, R, G;                   // chunk-causal variant (CC > 0): chunk length, chunk count, the token split
  int LW;                               // local-window variant: window in tokens on either side of the query tile
  int has_linear, P, act;
  int64_t sb, sh, sn;
  float scale_log2e;
};

// Pieces of the epilogue of one 32-query column block (Eq. "hybrid"): g = phi_q(q), n = g S, e = g.z,
// y = (a + n) / (l + e); `o` holds a^T (d x queries) as C tiles, `lsum` this lane's half of l.

// bf16 copy of the activated tiles: the B operand ("chained" order) of the contraction with the state
template <int FB>
static __device__ __forceinline__ void round_tiles(const f32x16 (&u)[FB], bf16x8 (&gb)[FB][2]) {
#pragma unroll
  for (int fb = 0; fb < FB; ++fb)
#pragma unroll
    for (int sp = 0; sp < 2; ++sp) {
      f32x8 t8;
#pragma unroll
      for (int i = 0; i < 8; ++i) t8[i] = u[fb][8 * sp + i];
      gb[fb][sp] = __builtin_convertvector(t8, bf16x8);
    }
}

// e = g.z with the bf16-rounded g, so that numerator and denominator see the same g (this lane's half)
template <int FB>
static __device__ __forceinline__ float dot_z(const bf16x8 (&gb)[FB][2], const float *zz, int g) {
  float e = 0.f;
#pragma unroll
  for (int fb = 0; fb < FB; ++fb)
#pragma unroll
    for (int sp = 0; sp < 2; ++sp)
#pragma unroll
      for (int i = 0; i < 8; ++i) e += static_cast<float>(gb[fb][sp][i]) * zz[32 * fb + crow(8 * sp + i, g)];
  return e;
}

// o^T += S^T g^T with S^T as hi + lo bf16 fragments (sth / stl: global through a descriptor, or LDS)
template <int D, int F, typename WP>
static __device__ __forceinline__ void contract_state(const bf16x8 (&gb)[F / 32][2], WP sth, WP stl, int lane,
                                                      f32x16 (&o)[D / 32]) {
  constexpr int RB = D / 32, FB = F / 32;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    f32x16 n;
#pragma unroll
    for (int x = 0; x < 16; ++x) n[x] = 0.f;
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
      for (int sp = 0; sp < 2; ++sp) {
        const int idx = (rb * FB + fb) * 2 + sp;
        n = mfma32(frag_at(stl, idx, lane), gb[fb][sp], n);
        n = mfma32(frag_at(sth, idx, lane), gb[fb][sp], n);
      }
#pragma unroll
    for (int x = 0; x < 16; ++x) o[rb][x] += n[x];
  }
}

// Store y = o * inv.  The C layout has one query per lane with 4 consecutive channels per register group, i.e.
// 8-byte pieces 256 bytes apart across lanes.  The tile goes through this wave's LDS staging area instead
// ([32 queries][channels of one pass], rows padded by 16 bytes) and leaves as 16-byte pieces with
// consecutive lanes on consecutive addresses of a row.
// Row denominators for a caller that differentiates the output (value distillation): lane r of the lower half
// holds the denominator of query q_first + r.
static __device__ __forceinline__ void store_den(const QueryArgs &a, int bh, int lane, float den, int q_first) {
  if (a.row_den && lane < 32 && q_first + lane < a.N) a.row_den[(int64_t)bh * a.N + q_first + lane] = den;
}

template <int D, bool F32>
static __device__ __forceinline__ void store_tile(const QueryArgs &a, int64_t base, int lane, const f32x16 (&o)[D / 32],
                                                  float inv, char *stage, int q_first) {
  constexpr int RB = D / 32;
  constexpr int PASSES = F32 ? 2 : 1;               // fp32 output is staged half a row at a time
  constexpr int DP = D / PASSES, ESZ = F32 ? 4 : 2;
  constexpr int PITCH = DP * ESZ + 16;              // bytes
  constexpr int CPR = DP * ESZ / 16;                // 16-byte pieces per staged row
  const int r = lane & 31, g = lane >> 5;
#pragma unroll
  for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
    for (int rbl = 0; rbl < RB / PASSES; ++rbl) {
      const int rb = pass * (RB / PASSES) + rbl;
#pragma unroll
      for (int x4 = 0; x4 < 4; ++x4) {
        const int dloc = 32 * rbl + 8 * x4 + 4 * g;
        f32x4 y = {o[rb][4 * x4] * inv, o[rb][4 * x4 + 1] * inv, o[rb][4 * x4 + 2] * inv, o[rb][4 * x4 + 3] * inv};
        if constexpr (F32) *reinterpret_cast<f32x4 *>(stage + r * PITCH + dloc * 4) = y;
        else *reinterpret_cast<bf16x4 *>(stage + r * PITCH + dloc * 2) = __builtin_convertvector(y, bf16x4);
      }
    }
    // the staging area is this wave's own and a wave's LDS instructions execute in order: no workgroup barrier, the
    // compiler only has to keep the reads behind the writes
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = lane; i < 32 * CPR; i += 64) {
      const int row = i / CPR, ch = i % CPR;
      if (q_first + row < a.N) {
        const f32x4 piece = *reinterpret_cast<const f32x4 *>(stage + row * PITCH + ch * 16);
        char *dst = static_cast<char *>(a.out) + (base + (int64_t)(q_first + row) * a.sn + pass * DP) * ESZ + ch * 16;
        *reinterpret_cast<f32x4 *>(dst) = piece;
      }
    }
    if (PASSES > 1) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
}

// The whole epilogue with every operand array in one place for its whole duration.
// ELDS: w2f / sth / stl sit in the ring and were requested when the loop ended (they land while layer 1 runs).
template <int D, int HD, int F, bool F32, bool ELDS, typename WP>
static __device__ __forceinline__ void query_epilogue(const QueryArgs &a, int bh, int h, int64_t base, int lane,
                                                      const bf16x8 (&qf)[D / 16], f32x16 (&o)[D / 32], float lsum,
                                                      WP w1f, WP w2f, WP sth, WP stl, char *stage, int q_first) {
  constexpr int FB = F / 32;
  const int g = lane >> 5;
  float den = xhalf_sum(lsum);
  if (a.has_linear) {
    const float *b1 = a.b1 ? a.b1 + (int64_t)h * HD : nullptr;
    const float *b2 = a.b2 ? a.b2 + (int64_t)h * F : nullptr;
    bf16x8 gb[FB][2];
    {
      bf16x8 h_hi[HD / 32][2], h_lo[HD / 32][2];
      feature_mlp_layer1<D, HD>(qf, w1f, b1, lane, g, h_hi, h_lo);
      if constexpr (ELDS) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
      }
      if constexpr (F > 128) {
        feature_layer2_phi<HD, F, false>(h_hi, h_lo, w2f, b2, lane, g, a.act, a.P, F / a.P, gb);
      } else {
        f32x16 u[FB];
        feature_mlp_layer2<HD, F>(h_hi, h_lo, w2f, b2, lane, g, u);
        feature_activation<FB>(u, g, a.act, a.P, F / a.P);
        round_tiles<FB>(u, gb);
      }
    }
    den += xhalf_sum(dot_z<FB>(gb, a.z + (int64_t)bh * F, g));
    contract_state<D, F>(gb, sth, stl, lane, o);
  }
  if constexpr (ELDS) {
    if (a.has_linear) __syncthreads();   // every wave is done with the operands in the ring: it becomes the staging area
  }
  store_den(a, bh, lane, den, q_first);
  store_tile<D, F32>(a, base, lane, o, 1.0f / den, stage, q_first);
}

// ------------------------------------------------------------------------------------------------
// query_kernel_ring: the softmax tile loop as a software pipeline.  NW waves, each owning one column block
// of 32 queries.
//
// K_S / V_S fragments travel global -> LDS with direct-to-LDS loads into a ring of NB 32-key blocks
// (no staging registers).  Loop step j handles key block j:
//   phase 1   S(j+1)^T = K(j+1) Q^T on the matrix cores   ||   softmax of S(j) on the vector ALU;
//             V(j) and K(j+2) fragments LDS -> registers (two K buffers alternate)
//   phase 2   O^T += V(j)^T P(j)^T                          ||   column maxima of S(j+1)
// Every block runs the same step, also the (at most one) step past the last block, whose logits are masked.
// The block for step j + LEAD (LEAD = NB - G) is requested at the top of step j; a barrier (after
// waiting for this wave's outstanding loads) closes every G-th step.  NB >= 2 G + 2 makes this safe:
// the slot being refilled was last read before the latest barrier every wave has passed, and a block
// is first read (as K(j+2)) at least one barrier after it was requested.
// LIN: the linear part arrives precomputed (maps too wide for the epilogue below); a variant of its own so that
// the usual kernel carries none of it.
// MODE 1: the chunk-causal variant, 2: the local-window variant; likewise variants of their own.
template <int D, int HD, int F, int NW, int NB, int G, bool F32, bool LIN = false, int MODE = 0>
__global__ __launch_bounds__(64 * NW, 2) void query_kernel_ring(QueryArgs a) {
  static_assert(G <= 2 && NB >= 2 * G + 2 && (NB & (NB - 1)) == 0, "ring too short for the barrier period");
  constexpr int KS = D / 16, RB = D / 32;
  constexpr int FRAG = D * 4;                 // bf16x8 per 32-key block per tensor
  constexpr int LEAD = NB - G, QT = 32 * NW;
  constexpr int WCH = FRAG / 64;              // 1 KiB wave-chunks per block per tensor
  __shared__ bf16x8 ring[2 * NB * FRAG];
  // after the loop each wave stages its 32-query output tile in its share of the ring
  static_assert(32 * ((D / (F32 ? 2 : 1)) * (F32 ? 4 : 2) + 16) <= 2 * NB * FRAG * 16 / NW, "staging tile too large");
  bf16x8 (*ring_k)[FRAG] = reinterpret_cast<bf16x8 (*)[FRAG]>(&ring[0]);
  bf16x8 (*ring_v)[FRAG] = reinterpret_cast<bf16x8 (*)[FRAG]>(&ring[NB * FRAG]);
  // Epilogue operands through LDS (one fetch per workgroup instead of one per wave) where they fit: the
  // layer-1 weights of phi_q in an area of their own, fetched at kernel start; the layer-2 weights and the
  // state (hi + lo) in the ring once the loop has ended.
  constexpr int NW1 = HD * D / 8, NW2 = F * HD / 8, NST = D * F / 8;   // bf16x8 per head / per (batch, head)
  constexpr bool ELDS = !LIN && NW == 8 && NW1 * 16 <= 32 * 1024 && (NW2 + 2 * NST) <= 2 * NB * FRAG &&
                        NW1 % (64 * NW) == 0 && NW2 % (64 * NW) == 0 && NST % (64 * NW) == 0;
  __shared__ bf16x8 w1_lds[ELDS ? NW1 : 1];
  // Wider maps: the operands do not fit at once, but the ring takes them in three rounds after the loop
  // (layer-1 weights + first half of the layer-2 weights, second half, state hi + lo).
  constexpr bool PHASED = !LIN && NW == 8 && !ELDS && NW1 <= NB * FRAG && NW2 / 2 <= NB * FRAG && NST <= NB * FRAG &&
                          NW1 % 64 == 0 && (NW2 / 2) % 64 == 0 && NST % 64 == 0 && (F / 32) % 2 == 0;

  const int per_xcd = (a.total_wg + 7) >> 3;
  int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  constexpr bool CAUSAL = MODE == 1;
  if constexpr (CAUSAL) logical = blockIdx.x;
  if (logical >= a.total_wg) return;
  int bh = logical / a.n_qtiles, qtile = logical % a.n_qtiles;
  if constexpr (CAUSAL) {
    // the work of a tile grows with its position: the longest tiles of every (batch, head) are started first, and
    // consecutive workgroups (which land on different XCDs) take tiles of the same length
    const int n_bh = a.total_wg / a.n_qtiles;
    bh = logical % n_bh;
    qtile = a.n_qtiles - 1 - logical / n_bh;
  }
  const int h = bh % a.H;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)h * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, kept scalar
  const int q0 = qtile * QT + w * 32;
  if constexpr (CAUSAL) {
    // chunk-causal variant: this tile lies inside causal chunk cc (chunks are whole query tiles); it sees the softmax
    // keys of the first cc + 1 chunks, which lead the compacted arrays, and the prefix state of chunk cc
    const int cc = (qtile * QT) / a.CC;
    const int64_t shift = (int64_t)bh * (a.n_cc - 1) + cc;
    a.NS = softmax_before(min((cc + 1) * a.CC, a.N), a.R, a.G);
    a.z += shift * F;
    a.st_hi += shift * (D * F / 8);
    a.st_lo += shift * (D * F / 8);
  }
  int kb_lo = 0;                            // first key block this tile reads (local-window variant)
  if constexpr (MODE == 2) {
    // local-window variant: the softmax keys are the tokens of the tiles qtile - w .. qtile + w (every token sits in
    // the compacted arrays, in order), the state is the one of the tokens outside that window
    const int w_t = a.LW / QT, lo_tile = max(qtile - w_t, 0);
    const int64_t shift = (int64_t)bh * (a.n_cc - 1) + qtile;
    kb_lo = lo_tile * (QT / 32);
    a.NS = min((qtile + w_t + 1) * QT, a.N) - lo_tile * QT;
    a.z += shift * F;
    a.st_hi += shift * (D * F / 8);
    a.st_lo += shift * (D * F / 8);
  }
  // n_chunks 1 KiB wave-chunks global -> LDS, dealt round-robin to the waves (direct-to-LDS loads, see below)
  auto stage_in = [&](const bf16x8 *gsrc, bf16x8 *ldst, int n_chunks) {
    const unsigned lane_off16 = lane * 16;
    for (int ch = w; ch < n_chunks; ch += NW) {
      const unsigned l = __builtin_amdgcn_readfirstlane(
          (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)(ldst + ch * 64));
      const bf16x8 *gp = gsrc + ch * 64;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(l), "v"(lane_off16), "s"(gp) : "memory");
    }
  };
  const int nblk = (a.NS + 31) >> 5;     // key blocks that hold at least one real key
  // layer-1 weights of phi_q: not needed before the epilogue, so with a softmax loop ahead they are requested only
  // once the loop's first key blocks have landed (nothing at the start of the workgroup waits for them)
  if constexpr (ELDS) {
    if (a.has_linear) stage_in(a.w1f + (int64_t)h * NW1, w1_lds, NW1 / 64);
  }

  bf16x8 qf[KS];
  {
    const int qi = min(q0 + r, a.N - 1);   // rows past the end repeat the last query and are not stored
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = load8<F32>(a.q, base + (int64_t)qi * a.sn + 16 * ks + 8 * g);
  }
  f32x16 o[RB];
  // m_true: exact running maximum c_i over the keys this lane has seen, i.e. over its half of every key block (the
  // two halves of a query column meet only when it matters: in the rare rescale and once after the loop).
  // m: the (possibly older) maximum the accumulators are currently expressed against, the same in both halves; it
  // follows m_true only when the gap would let exponentials exceed 2^kLazy.
  constexpr float kLazy = 8.0f;
  float m = -INFINITY, m_true = -INFINITY, lsum = 0.f;
  // Row sums of P on the matrix cores (the issue port, not the matrix core, is what the loop's vector work crowds): a 16x16x32 product of a constant 0/1 matrix with the very B operand of P V.
  // Its lane layout (column = lane % 16, contraction group = lane / 16) sees the 32-query operand as two interleaved
  // 16-query ones: groups 0, 2 hold query lane % 16, groups 1, 3 hold query 16 + lane % 16.  Row 0 of the constant
  // matrix selects groups 0, 2 and row 4 groups 1, 3, so register 0 of lane r < 32 receives the whole sum of query r
  // (both halves of its keys) and the upper 32 lanes receive zero, which is what the final cross-half sum expects.
  f32x4 lacc = {0.f, 0.f, 0.f, 0.f};
  bf16x8 sel;
  {
    const int row = lane & 15, kq = lane >> 4;
    const __bf16 one = static_cast<__bf16>(((row == 0 && (kq & 1) == 0) || (row == 4 && (kq & 1) == 1)) ? 1.0f : 0.0f);
    sel = bf16x8{one, one, one, one, one, one, one, one};
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int x = 0; x < 16; ++x) o[rb][x] = 0.f;

  if (nblk > 0) {
    const bf16x8 *ksrc = a.ks_frag + ((int64_t)bh * a.n_kblocks + kb_lo) * FRAG;
    const bf16x8 *vsrc = a.vs_frag + ((int64_t)bh * a.n_kblocks + kb_lo) * FRAG;
    const int kb_last = a.n_kblocks - 1 - kb_lo;
    const unsigned lane_off = lane * 16;
    // block b: global -> ring slot b % NB with direct-to-LDS loads; one instruction moves 64 lanes x 16 B
    // = one 1 KiB wave-chunk (LDS address = M0 + 16 * lane, global address = scalar base + 16 * lane), and
    // the wave-chunks of a block are dealt round-robin to the waves.  Issued as inline asm so that the
    // compiler does not make later LDS reads of OTHER ring slots wait for it; completion is awaited
    // explicitly before each barrier.
    auto request = [&](int b) {
      const int slot = b & (NB - 1);
#pragma unroll
      for (int i = 0; i < (WCH + NW - 1) / NW; ++i) {
        const int ch = i * NW + w;
        if (WCH % NW == 0 || ch < WCH) {
          const unsigned lk = __builtin_amdgcn_readfirstlane(
              (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)(&ring_k[slot][ch * 64]));
          const unsigned lv = __builtin_amdgcn_readfirstlane(
              (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)(&ring_v[slot][ch * 64]));
          const bf16x8 *gk = ksrc + (int64_t)b * FRAG + ch * 64;
          const bf16x8 *gv = vsrc + (int64_t)b * FRAG + ch * 64;
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\t"
                       "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %4"
                       :: "s"(lk), "v"(lane_off), "s"(gk), "s"(lv), "s"(gv) : "memory");
        }
      }
    };
    // Barrier that closes a group of G steps.  Everything this wave requested must have landed before
    // the other waves may read it, except the newest blocks: the steps up to the next barrier read no
    // block beyond (closing step) + G + 2, so in the steady state the requests of the last
    // NB - 2G - 2 steps may stay in flight (loads retire in order).
    constexpr int IPB = 2 * ((WCH + NW - 1) / NW);          // load instructions per block per wave
    constexpr int INFLIGHT = (NB - 2 * G - 2) * IPB;
    auto ring_barrier = [&](auto steady) {
      if constexpr (decltype(steady)::value && INFLIGHT > 0) {
        static_assert(INFLIGHT <= 15, "vmcnt immediate too large");
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(INFLIGHT) : "memory");
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
      __syncthreads();
    };
    // Every step of the loop below runs the same code, also past the last block (its logits are masked
    // and its weights are zero), so every ring slot must hold finite data before it is read: requests past
    // the end re-fetch the last block of the (zero padded) fragment arrays.
    for (int b = 0; b < LEAD; ++b) request(min(b, kb_last));
    ring_barrier(std::false_type{});

    const float c = a.scale_log2e;
    const float lazy_gap = kLazy / c;                   // the threshold in units of the raw logits
    float mc = 0.f;                                     // m c, kept beside m (it changes only in the rare rescale)
    bf16x8 k_a[KS], k_b[KS], vf[RB][2];
    f32x16 s_a, s_b;
    auto load_k = [&](int b, bf16x8 (&dst)[KS]) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) dst[ks] = ring_k[b & (NB - 1)][ks * 64 + lane];
    };
    // logits of block b that are zero padding (keys >= NS) must not take part
    auto mask_tail = [&](f32x16 &s, int b) {
      if ((b + 1) * 32 > a.NS) {
#pragma unroll
        for (int x = 0; x < 16; ++x) s[x] = (b * 32 + crow(x, g) >= a.NS) ? -INFINITY : s[x];
      }
    };
    // Running maximum c_i over the blocks seen so far.  The accumulators follow it lazily: they are
    // rescaled only when some row's maximum has moved more than kLazy (in log2 units) past the reference
    // they are expressed against, which keeps every exponential below 2^kLazy; the exact c_i is restored
    // once after the loop.
    auto fold_max = [&](const f32x16 &s) {
      float t = m_true;                                 // the running maximum rides along as a seventeenth value
#pragma unroll
      for (int x = 0; x < 16; ++x) t = fmaxf(t, s[x]);
      m_true = t;
      if (__any(m_true - m > lazy_gap)) {
        m_true = xhalf_max(m_true);
        const float alpha = fast_exp2((m - m_true) * c);
        lacc[0] *= alpha;                                 // registers 1 - 3 hold rows of zeros
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int x = 0; x < 16; ++x) o[rb][x] *= alpha;
        m = m_true;
        mc = m * c;
      }
    };

    // prologue: S(0), its maximum, and the K fragments of block 1
    load_k(0, k_b);
#pragma unroll
    for (int x = 0; x < 16; ++x) s_a[x] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s_a = mfma32(k_b[ks], qf[ks], s_a);
    mask_tail(s_a, 0);
    fold_max(s_a);
    load_k(1, k_a);

    // One step.  On entry s_cur = S(j)^T (masked), m already covers block j, k_cur holds K(j+1).  Blocks past
    // the last real one are processed like any other: their logits are masked to -inf (weights exactly 0).
    // All LDS reads of a step are issued during phase 1, a phase or more ahead of their use: V(j) for
    // phase 2 of this step, K(j+2) (into the other K buffer) for phase 1 of the next.
    // MASK: block j + 1 may hold padding keys (or lie past the end).
    auto step = [&](int j, f32x16 &s_cur, f32x16 &s_nxt, bf16x8 (&k_cur)[KS], bf16x8 (&k_nxt)[KS], auto mask_c) {
      constexpr bool MASK = decltype(mask_c)::value;
      request(min(j + LEAD, kb_last));
      const bf16x8 *vsrc_lds = ring_v[j & (NB - 1)], *ksrc_lds = ring_k[(j + 2) & (NB - 1)];
      // phase 1: S(j+1)^T on the matrix cores, exponentials of S(j)^T on the VALU
      bf16x8 pb[2];
#pragma unroll
      for (int x = 0; x < 16; ++x) s_nxt[x] = 0.f;
      constexpr int PER = 16 / KS;   // logits per matrix instruction: 2 for d = 128, 4 for d = 64
      constexpr int QTR = KS / 4 > 0 ? KS / 4 : 1;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        // LDS reads, a quarter of the step's sixteen fragments at a time
        if (ks == 0) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) vf[rb][0] = vsrc_lds[(rb * 2 + 0) * 64 + lane];
        } else if (ks == QTR) {
#pragma unroll
          for (int t = 0; t < KS / 2; ++t) k_nxt[t] = ksrc_lds[t * 64 + lane];
        } else if (ks == 2 * QTR) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) vf[rb][1] = vsrc_lds[(rb * 2 + 1) * 64 + lane];
        } else if (ks == 3 * QTR) {
#pragma unroll
          for (int t = KS / 2; t < KS; ++t) k_nxt[t] = ksrc_lds[t * 64 + lane];
        }
        s_nxt = mfma32(k_cur[ks], qf[ks], s_nxt);
        // a slice of the exponentials rides along with every matrix instruction
#pragma unroll
        for (int i = 0; i < PER; ++i) {
          const int x = ks * PER + i;
          s_cur[x] = fast_exp2(__builtin_fmaf(s_cur[x], c, -mc));
        }
        // once a half of the block is exponentiated it is rounded to bf16 (the B operand of P V) and its
        // row-sum contribution is taken from the rounded values, so that numerator and denominator see the
        // same weights
        if (ks == KS / 2 - 1 || ks == KS - 1) {
          const int sp = ks == KS - 1;
          f32x8 p8;
#pragma unroll
          for (int i = 0; i < 8; ++i) p8[i] = s_cur[8 * sp + i];
          pb[sp] = __builtin_convertvector(p8, bf16x8);
          lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, pb[sp], lacc, 0, 0, 0);
        }
      }
      // phase 2: O^T += V(j)^T P(j)^T on the matrix cores; the column maxima of S(j+1)^T on the VALU
#pragma unroll
      for (int sp = 0; sp < 2; ++sp)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) o[rb] = mfma32(vf[rb][sp], pb[sp], o[rb]);
      if constexpr (MASK) mask_tail(s_nxt, j + 1);
      fold_max(s_nxt);
    };
    using T = std::true_type;
    using Fa = std::false_type;
    // two steps per trip (the two S buffers swap roles); an odd block count adds one all-masked step.
    // Trips whose blocks j + 1, j + 2 consist of real keys only skip the padding mask.
    const int n_full = a.NS >> 5;
    int j = 0;
    for (; j + 2 < n_full; j += 2) {
      step(j, s_a, s_b, k_a, k_b, Fa{});
      if (G == 1) ring_barrier(T{});
      step(j + 1, s_b, s_a, k_b, k_a, Fa{});
      ring_barrier(T{});
    }
    for (; j < nblk; j += 2) {
      step(j, s_a, s_b, k_a, k_b, T{});
      if (G == 1) ring_barrier(T{});
      step(j + 1, s_b, s_a, k_b, k_a, T{});
      ring_barrier(T{});
    }
    ring_barrier(Fa{});   // everything landed and read: the ring is free for the epilogue
    // express the accumulators against the exact c_i (Eq. "hybrid": the largest softmax weight is 1)
    m_true = xhalf_max(m_true);
    const float alpha = fast_exp2((m - m_true) * c);
    lsum = lacc[0] * alpha;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int x = 0; x < 16; ++x) o[rb][x] *= alpha;
  }
  char *stage = reinterpret_cast<char *>(&ring[0]) + w * (2 * NB * FRAG * 16 / NW);
  if constexpr (LIN) {
    // linear part computed by the wide-map passes: add it to the accumulators, which share its register layout
    float den = xhalf_sum(lsum);
    const int tb = q0 >> 5;
    if (tb < a.n_tb) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int x4 = 0; x4 < 4; ++x4) {
          const f32x4 t = a.lin[((((int64_t)bh * a.n_tb + tb) * RB + rb) * 4 + x4) * 64 + lane];
#pragma unroll
          for (int j = 0; j < 4; ++j) o[rb][4 * x4 + j] += t[j];
        }
      den += a.lin_e[(int64_t)bh * a.N + min(q0 + (lane & 31), a.N - 1)];
    }
    store_den(a, bh, lane, den, q0);
    store_tile<D, F32>(a, base, lane, o, 1.0f / den, stage, q0);
    return;
  }
  const bf16x8 *w1g = a.w1f + (int64_t)h * NW1;
  const bf16x8 *w2g = a.w2f + (int64_t)h * NW2;
  const bf16x8 *sthg = a.st_hi + (int64_t)bh * NST;
  const bf16x8 *stlg = a.st_lo + (int64_t)bh * NST;
  if constexpr (ELDS) {
    typedef lds_frag_ptr lds_ptr;
    if (a.has_linear) {
      stage_in(w2g, &ring[0], NW2 / 64);
      stage_in(sthg, &ring[NW2], NST / 64);
      stage_in(stlg, &ring[NW2 + NST], NST / 64);
      // the layer-1 weights were requested at kernel start; with no key block at all nothing has waited for them yet
      asm volatile("s_waitcnt vmcnt(%0)" :: "n"((NW2 + 2 * NST) / 64 / NW) : "memory");
      __syncthreads();
    }
    query_epilogue<D, HD, F, F32, true>(a, bh, h, base, lane, qf, o, lsum, (lds_ptr)&w1_lds[0], (lds_ptr)&ring[0],
                                        (lds_ptr)&ring[NW2], (lds_ptr)&ring[NW2 + NST], stage, q0);
  } else if constexpr (PHASED) {
    typedef lds_frag_ptr lds_ptr;
    constexpr int FB = F / 32, HB = HD / 32, HALF = NB * FRAG;
    const int g = lane >> 5;
    float den = xhalf_sum(lsum);
    auto landed = [&]() {                       // this wave's requests have landed, and so have everybody's
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    };
    if (a.has_linear) {
      const float *b1 = a.b1 ? a.b1 + (int64_t)h * HD : nullptr;
      const float *b2 = a.b2 ? a.b2 + (int64_t)h * F : nullptr;
      bf16x8 gb[FB][2];
      stage_in(w1g, &ring[0], NW1 / 64);
      stage_in(w2g, &ring[HALF], NW2 / 2 / 64);
      landed();
      {
        PhiState<FB> st;
        bf16x8 h_hi[HB][2], h_lo[HB][2];
        feature_mlp_layer1<D, HD>(qf, (lds_ptr)&ring[0], b1, lane, g, h_hi, h_lo);
        feature_layer2_phi_tiles<HD, F, 0, FB / 2, false>(h_hi, h_lo, (lds_ptr)&ring[HALF], 0, b2, lane, g, a.act, a.P,
                                                          F / a.P, st, gb);
        __syncthreads();                        // every wave is done with W1 and the first half of W2
        stage_in(w2g + NW2 / 2, &ring[0], NW2 / 2 / 64);
        landed();
        feature_layer2_phi_tiles<HD, F, FB / 2, FB, false>(h_hi, h_lo, (lds_ptr)&ring[0], (FB / 2) * HB * 2, b2, lane, g,
                                                           a.act, a.P, F / a.P, st, gb);
        feature_phi_finish<F>(st, a.act, a.P, F / a.P, gb);
      }
      den += xhalf_sum(dot_z<FB>(gb, a.z + (int64_t)bh * F, g));
      __syncthreads();                          // second half of W2 no longer needed
      stage_in(sthg, &ring[0], NST / 64);
      stage_in(stlg, &ring[HALF], NST / 64);
      landed();
      contract_state<D, F>(gb, (lds_ptr)&ring[0], (lds_ptr)&ring[HALF], lane, o);
      __syncthreads();                          // the ring becomes the staging area of the stores
    }
    store_den(a, bh, lane, den, q0);
    store_tile<D, F32>(a, base, lane, o, 1.0f / den, stage, q0);
  } else {
    // the operands do not fit next to the ring: read in place (L2-resident, per head / per (batch, head))
    query_epilogue<D, HD, F, F32, false>(a, bh, h, base, lane, qf, o, lsum, global_frags(w1g, NW1 * 16),
                                         global_frags(w2g, NW2 * 16), global_frags(sthg, NST * 16),
                                         global_frags(stlg, NST * 16), stage, q0);
  }
}

hipError_t launch_query(const Plan &pl, const void *q, const ha_feature_map *phi_q, void *out, float *row_den, void *ws,
                        hipStream_t st, const WidePlan *wide) {
  QueryArgs a;
  a.q = q;
  a.out = out;
  a.row_den = row_den;
  a.lin = wide ? ws_ptr<f32x4>(ws, wide->off_lin) : nullptr;
  a.lin_e = wide ? ws_ptr<float>(ws, wide->off_e) : nullptr;
  a.n_tb = wide ? wide->n_tb_q : 0;
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
  a.CC = pl.CC; a.n_cc = pl.n_cc; a.R = pl.R; a.G = pl.G; a.LW = pl.LW;
  a.n_ktiles = pl.n_ktiles; a.n_kblocks = pl.n_kblocks;
  a.has_linear = pl.NL > 0; a.P = pl.P; a.act = pl.act_q;
  a.sb = pl.sb; a.sh = pl.sh; a.sn = pl.sn;
  a.scale_log2e = pl.scale * kLog2e;
  // block_size 128: 8 waves x 32 queries, ring of 8 key blocks, barrier every 64 keys (one workgroup per CU);
  // block_size 64: 4 waves x 32 queries, ring of 4 key blocks, barrier every 32 keys (two workgroups per CU).
  const bool big = pl.KT == 128;
  a.n_qtiles = pl.n_qtiles;
  a.total_wg = a.n_qtiles * pl.B * pl.H;
  dim3 grid(((a.total_wg + 7) / 8) * 8);
#define HA_QUERY(DD, HH, FF, F32) \
  do { \
    if (pl.LW > 0) { \
      if (big) query_kernel_ring<DD, HH, FF, 8, 8, 2, F32, false, 2><<<grid, 512, 0, st>>>(a); \
      else query_kernel_ring<DD, HH, FF, 4, 4, 1, F32, false, 2><<<grid, 256, 0, st>>>(a); \
    } else if (pl.CC > 0) { \
      if (big) query_kernel_ring<DD, HH, FF, 8, 8, 2, F32, false, 1><<<grid, 512, 0, st>>>(a); \
      else query_kernel_ring<DD, HH, FF, 4, 4, 1, F32, false, 1><<<grid, 256, 0, st>>>(a); \
    } else { \
      if (big) query_kernel_ring<DD, HH, FF, 8, 8, 2, F32><<<grid, 512, 0, st>>>(a); \
      else query_kernel_ring<DD, HH, FF, 4, 4, 1, F32><<<grid, 256, 0, st>>>(a); \
    } \
  } while (0)
  if (wide) {
    if (big) {
      if (pl.f32) query_kernel_ring<128, 128, 128, 8, 8, 2, true, true><<<grid, 512, 0, st>>>(a);
      else query_kernel_ring<128, 128, 128, 8, 8, 2, false, true><<<grid, 512, 0, st>>>(a);
    } else {
      if (pl.f32) query_kernel_ring<128, 128, 128, 4, 4, 1, true, true><<<grid, 256, 0, st>>>(a);
      else query_kernel_ring<128, 128, 128, 4, 4, 1, false, true><<<grid, 256, 0, st>>>(a);
    }
  }
  else if (pl.D == 64) { if (pl.f32) HA_QUERY(64, 64, 64, true); else HA_QUERY(64, 64, 64, false); }
  else if (pl.HD == 128) { if (pl.f32) HA_QUERY(128, 128, 128, true); else HA_QUERY(128, 128, 128, false); }
  else { if (pl.f32) HA_QUERY(128, 256, 256, true); else HA_QUERY(128, 256, 256, false); }
#undef HA_QUERY
  return hipGetLastError();
}

}  // namespace ha
