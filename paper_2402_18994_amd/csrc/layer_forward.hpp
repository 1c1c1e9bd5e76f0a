// Forward pass of a whole feed-forward LIF layer in one launch (Eq. 1-2): currents
// I = S_below W, the scan over time, V and S stored; I never goes to memory.
//
// As separate launches the product writes I (4 bytes per element) and the scan reads it back:
// at 128 neurons that round trip is most of both kernels' traffic, and at 32 768 chains the
// scan has two wavefronts per compute unit which each issue a load and two stores per step.
// Here a workgroup owns one sample and BN = 64 or 128 of the layer's neurons (a layer of ld
// neurons is cut in ld / BN parts; the parts of a sample run on the same XCD and share its
// spike rows in that L2).  Per block of 128 steps:
//   1. product: the 128 rows (t, b) of the spike tensor below times the rounded weights, on
//      the streamed pipeline of the large current products (operands straight into LDS,
//      three stages of 64, see gemm_stream.hpp); the rows of the tile are the sample's time steps,
//      so W passes through the workgroup once per block and the spikes once in all;
//   2. the 128 x BN tile of currents goes to LDS (the stages are free by then);
//   3. scan: BN / 64 wavefronts hold one neuron per lane and walk the 128 steps on LDS: read
//      I_t (16 steps ahead), write V_t back in place.  The spike decision is taken without a
//      compare: s = clamp((V - theta) 2^100) is exactly 1 when V > theta and 0 otherwise
//      (for theta in [2^-60, 2^26]: the difference of two floats, when positive, is at least
//      2^-24 theta, and the scaling is exact in the fused multiply-add), and V' = (beta V + I)
//      - theta s is the value the plain scan computes.  Compare, select and subtract cost 57
//      cycles per step as a dependent chain (the compare's result travels through a scalar
//      register); the two fused multiply-adds take 35;
//   4. store: all four wavefronts write V as whole rows, 16 bytes per lane, and S as 16
//      neurons per lane, decided again from the stored V (the same exact comparison);
//   5. (last spiking layer of 128 neurons, at most 32 padded classes) the readout's currents
//      J = S W_out of the block, eight 32x32x16 MFMAs per wavefront on the spikes in LDS: no
//      product launch for the readout;
//   6. (same case) the readout itself: the LI scan of the block in eight segments of 16 steps
//      (linear in the state, so segments are integrated from zero, chained, and integrated
//      again from their true entry state), the maximum over time or the integral, and after
//      the last block softmax cross-entropy, dz and the readout's current gradients in closed
//      form per segment: no launch for the readout at all.
// The potential is carried in the scanning lanes' registers from block to block.
// Rows past T read as zero and are not stored; columns of W past the fan-in are zero.
// Two consecutive layers of exactly 128 neurons can share the launch (NL = 2): per block the
// workgroup runs steps 1 to 4 for the lower layer, waits until its spike stores are
// acknowledged, and runs them again for the upper layer on the rows it has just written.
// PACKED: the bottom layer of the launch reads the input raster packed along time (eight steps
// per byte, Section 2.1.4): the 16 packed rows of the sample's block sit in LDS for the whole
// product and are unpacked between the fragment read and the MFMA; the stages carry W alone.
// TS = 2 (blocks of 64 steps, TMV = 1): two workgroups share a sample and take its blocks in turn.
// Only the scan needs the block before it; the product of block k + 1 (most of a block's time)
// does not, so it runs on the other workgroup while block k is still being scanned.  What the
// scan of block k + 1 needs - the potentials after block k, and for the readout its state, the
// running maximum, its step and the running sum - goes through a small buffer in memory: written
// with device-scope accesses, the writer waits for its stores to be acknowledged and then raises
// a flag, the reader polls the flag (a bounded number of times: if the flag never comes, the
// error bit 1 is set and the kernel still ends) and reads with device-scope loads.  The workgroup
// of a sample's first block has the lower id, so it is never dispatched after the one that
// waits for it.
#pragma once
#include "gemm_stream.hpp"

namespace snn {

// One layer of the launch: operands and results.
struct LayerForwardOp {
  const uint8_t *P;        // spikes below [T*B][ldp], bytes 0/1 (PACKED, bottom layer: [ceil(T/8)*B][ldp], eight steps per byte)
  int ldp, kc;             // row length, fan-in
  unsigned p_bytes;
  const uint16_t *Q;       // rounded W^T [ld or more][ldq] bfloat16, zero beyond the fan-in and fan-out
  int ldq;
  unsigned q_bytes;
  float *V;                // [T*B][ld]
  uint8_t *S;              // [T*B][ld]
  const float *beta_v;     // [ld]
};

struct LayerForwardArgs {
  // The layers of the launch, bottom up.  More than one (kernel variants NL > 1, layers of
  // exactly 128 padded neurons): op[i + 1].P is op[i].S, and a workgroup takes its sample
  // through all of them block by block, reading back the spikes it has just stored.
  LayerForwardOp op[2];
  float theta;             // in [2^-60, 2^26]
  int T, B, ld;            // ld: a multiple of the workgroup's 64 or 128 neurons
  int nt_store;            // V and S stream past the caches
  // Readout currents J = S W_out, formed from the block's spikes while they are in LDS (only
  // the kernel variant for a last spiking layer of exactly 128 padded neurons uses these):
  float *J;                // [T*B][ldj], ldj a multiple of 8, at most 32
  int ldj;
  const uint16_t *Qr;      // rounded W_out^T [32 or more rows: class][ldqr: neuron] bfloat16, zero beyond the classes
  int ldqr;
  unsigned qr_bytes;
  // ... and the whole readout (variants READOUT >= 2): LI scan, max over time or integral,
  // softmax cross-entropy and the readout's current gradients, as readout_loss_kernel computes them
  float *Y;                // [T*B][ldj] readout trace
  float *z;                // [B][ldj] logits
  int *tstar;              // [B][ldj] first maximising step
  const int *labels;       // [B]
  float *loss_b;           // [B] per-sample loss
  float *dz;               // [B][ldj]
  int *err;                // flag: bit 0 = label out of range
  uint32_t *dJ;            // [T*B][ldj] hi/lo words
  const float *beta_r;     // [ldj] decays of the readout
  int C;                   // classes
  // Time-split variants (TS = 2): per sample SNN_HAND_BYTES of hand-over space.  Dwords 0..15:
  // flags (one per layer of the launch, [2]: the readout), each holding epoch * 1024 + the number of
  // blocks whose state has been published; then per layer two slots of 128 potentials; then two
  // slots of 256 x 4 dwords of readout state (state, running maximum, its step, running sum per
  // thread).  `epoch` grows with every launch, so flags never have to be cleared.
  uint32_t *hand;
  int epoch;
};
#define SNN_HAND_BYTES 12288
constexpr int HAND_V = 16, HAND_R = 16 + 2 * 2 * 128;      // dword offsets of the potential slots and the readout slots

__device__ __forceinline__ void hand_store(uint32_t *p, uint32_t x) {
  __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t hand_load(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// One thread polls until the flag has reached `want` (wrap-safe), at most 2^20 times (about a
// second); then sets bit 1 of the error word and goes on, so that the grid always drains.
__device__ __forceinline__ void hand_wait(const uint32_t *flag, uint32_t want, int *err) {
  int n = 0;
  while ((int)(hand_load(flag) - want) < 0) {
    if (++n >= (1 << 20)) { atomicOr(err, 2); break; }
    __builtin_amdgcn_s_sleep(2);
  }
}

// READOUT: 0 none; 1 the launch also forms the readout's currents J; 2 and the LI scan, the
// maximum over time, the loss and dJ; 3 the same with the integral loss.
//
// The work of one workgroup: NL layers of the launch from layer LI0 on, for the blocks half, half +
// TS, ... of sample b (TM: 64 TM steps per block).  ROLE: 0 the workgroup depends on no other (or,
// TS = 2, on the one that takes the sample's other blocks); 1 it runs the lower layer of a pair and
// tells the workgroup of the upper layer how many 64-step chunks of its spikes have reached memory;
// 2 it runs the upper layer and waits for the chunk of each of its blocks (see the kernel below).
template <int TN, int NS, int READOUT, int NL, bool PACKED, int TS, int TM, int LI0, int ROLE>
__device__ __forceinline__ void lif_layer_forward_body(const LayerForwardArgs &a, char *lds, float (*x_e)[8][32],
                                                       float (*x_best)[32], int (*x_tb)[32], const int b,
                                                       const int part, const int parts, const int half) {
  constexpr bool LOSS = READOUT >= 2, INTEGRAL = READOUT == 3;
  constexpr int JP = 36;                              // floats between rows of the BM x 32 readout tile in LDS
  typedef SpikeTile<2, 2, TM, TN, NS> Tile;
  constexpr int WN = 2, BM = Tile::BM, BN = Tile::BN, PI = Tile::PI, QI = Tile::QI, KS = Tile::KSTAGE;
  constexpr int SEG = BM / 8;                         // steps per segment of the readout scan (eight segments per block)
  static_assert((BM == 128 || BM == 64) && (BN == 64 || BN == 128), "128 or 64 steps x 64 or 128 neurons");
  static_assert(ROLE == 0 || (TS == 1 && NL == 1 && BM == (ROLE == 1 ? 128 : 64)), "a pair of layers on two workgroups");
  constexpr int CP = BN * 4 + 16;                     // bytes between time rows of the current tile in LDS
  constexpr int HAND_PAIR = 3;                        // flag of a pair of layers on two workgroups: chunks of 64 steps stored

  const int nblocks = (a.T + BM - 1) / BM;
  uint32_t *const hand = TS == 2 || ROLE ? a.hand + ((size_t)b * parts + part) * (SNN_HAND_BYTES / 4) : nullptr;
  const uint32_t hand_base = (uint32_t)a.epoch * 1024u;
  const int n0 = part * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN, h = lane >> 5;
  float beta[NL], v[NL];                              // decay and potential of neuron n0 + tid % BN, per layer
#pragma unroll
  for (int li = 0; li < NL; ++li) {
    beta[li] = a.op[li + LI0].beta_v[n0 + tid % BN];
    v[li] = 0.f;
  }
  const float theta = a.theta;
  const float big = 0x1p100f, mtheta_big = -theta * 0x1p100f, mtheta = -theta;

  // Readout state of class tid % 32 (variants with the loss)
  const float beta_r = LOSS && (tid & 31) < a.ldj ? a.beta_r[tid & 31] : 0.f;
  float bseg = beta_r;                                // beta^SEG
#pragma unroll
  for (int i = 1; i < SEG; i *= 2) bseg *= bseg;
  float y_in = 0.f, best = -INFINITY, ysum = 0.f;
  int lab = LOSS ? a.labels[b] : 0;                   // (asked for here: the epilogue would wait a memory round trip for it)
  int tb = 0, par = 0;

  for (int blk = half; blk < nblocks; blk += TS) {
   const int t0 = blk * BM;
   static_for<NL>([&](auto LI) {
    constexpr int li = decltype(LI)::value;
    constexpr bool last = li == NL - 1;
    const LayerForwardOp &op = a.op[li + LI0];
    const int nk = (op.kc + KS - 1) / KS;
    const u32x4 rp = raw_rsrc(op.P, op.p_bytes), rq = raw_rsrc(op.Q, op.q_bytes);
    const rsrc_t rV = make_rsrc(op.V, (unsigned)a.T * a.B * a.ld * 4u), rS = make_rsrc(op.S, (unsigned)a.T * a.B * a.ld);
    int qv[QI];
#pragma unroll
    for (int q = 0; q < QI; ++q) {
      const int row = Tile::q_row(wave, lane, q);
      qv[q] = ((n0 + row) * op.ldq + Tile::q_chunk(row, lane) * 8) * 2;
    }
    // 1. product (the upper layer of a pair on two workgroups: once the block's rows below are in memory)
    if (ROLE == 2) {
      if (tid == 0) hand_wait(hand + HAND_PAIR, hand_base + blk + 1, a.err);
      __syncthreads();
    }
    int pv[PI];
#pragma unroll
    for (int q = 0; q < PI; ++q) {
      const int row = Tile::p_row(wave, lane, q);
      pv[q] = row < BM && t0 + row < a.T ? ((t0 + row) * a.B + b) * op.ldp + Tile::p_unit(row, lane) * 16 : OOB;
    }
    f32x16 acc[TM][TN];
    if constexpr (PACKED && li + LI0 == 0) {
      PackedRows pk;
      pk.rsrc = make_rsrc(op.P, op.p_bytes);
      pk.base = ((t0 >> 3) * a.B + b) * op.ldp;
      pk.row_stride = a.B * op.ldp;
      pk.rows = ((a.T + 7) >> 3) - (t0 >> 3);
      pk.kbytes = op.ldp;
      Tile::template run<true>(lds, rp, rq, pv, qv, nk, wave, lane, acc, &pk);
    } else {
      Tile::run(lds, rp, rq, pv, qv, nk, wave, lane, acc);
    }

    // 2. The MFMAs take Q as their first operand, so a tile comes out transposed: the lane
    // holds time row (lane & 31) and register r neuron 8*(r/4) + 4*(lane/32) + (r%4).
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          u32x4 x;
          x.x = __float_as_uint(acc[i][j][4 * q]);
          x.y = __float_as_uint(acc[i][j][4 * q + 1]);
          x.z = __float_as_uint(acc[i][j][4 * q + 2]);
          x.w = __float_as_uint(acc[i][j][4 * q + 3]);
          const int row = (wm * TM + i) * 32 + (lane & 31), col = (wn * TN + j) * 32 + 8 * q + 4 * h;
          *(u32x4 *)(lds + row * CP + col * 4) = x;
        }
    if (TS == 2 && blk > 0 && tid == 0) hand_wait(hand + li, hand_base + blk, a.err);   // the block before has been scanned
    __syncthreads();

    // Readout variant: W_out^T as the first MFMA operand, lane -> class (lane & 31), neurons
    // 16 kk + 8 h .. +7.  Asked for here, once per block, so that the fragments arrive under the scan
    // and do not occupy 32 registers during the products.
    bf16x8 wr[READOUT && last ? 8 : 1];
    if constexpr (READOUT && last) {
      const rsrc_t rQ = make_rsrc(a.Qr, a.qr_bytes);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        wr[kk] = __builtin_bit_cast(bf16x8, ld_b128(rQ, ((lane & 31) * a.ldqr + 16 * kk + 8 * h) * 2, 0));
    }

    // 3. scan and store.  The wavefronts that hold no neuron (256 - BN threads) store what the scan
    // has finished, 16 steps behind it: after every 16 steps a barrier, behind which they read the
    // 16 rows of potentials back from the tile and write V (BN/4 pieces of 16 bytes per row) and S
    // (BN/16 pieces of 16 neurons per row, decided from V as in the scan) while the scan goes on
    // with the next rows.  (Steps past T run on zero currents; nothing of them is stored, and v is
    // not used after the last block.)
    constexpr int U = 16;
    if (wave < BN / 64) {
      if (TS == 2 && blk > 0) v[li] = __uint_as_float(hand_load(hand + HAND_V + (li * 2 + ((blk - 1) & 1)) * 128 + tid));
      float *cell = (float *)(lds + tid * 4);
      float nxt[U];
#pragma unroll
      for (int u = 0; u < U; ++u) nxt[u] = cell[u * (CP / 4)];
      for (int s0 = 0; s0 < BM; s0 += U) {
        // The currents of the next 16 steps are read before the 16 steps at hand are taken
        // (the empty asm keeps the reads here, not next to their use).
        float cur[U];
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = nxt[u];
        if (s0 + U < BM) {
#pragma unroll
          for (int u = 0; u < U; ++u) nxt[u] = cell[(s0 + U + u) * (CP / 4)];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) asm volatile("" : "+v"(cur[u]));
#pragma unroll
        for (int u = 0; u < U; ++u) {
          cell[(s0 + u) * (CP / 4)] = v[li];
          float s;                                    // 1 if v > theta, else 0
          asm("v_fma_f32 %0, %1, %2, %3 clamp" : "=v"(s) : "v"(v[li]), "v"(big), "v"(mtheta_big));
          v[li] = __builtin_fmaf(mtheta, s, __builtin_fmaf(beta[li], v[li], cur[u]));
        }
        __syncthreads();                              // rows s0 .. s0+15 hold potentials
        // (the storing wavefronts pass this barrier after the rows before s0 and, at the end of a
        // 64-step chunk, after the acknowledgement of their stores)
        if (ROLE == 1 && s0 > 0 && s0 % 64 == 0 && tid == 0) hand_store(hand + HAND_PAIR, hand_base + (t0 + s0) / 64);
      }
      if (TS == 2 && blk + 1 < nblocks) {             // hand the potentials on to the workgroup of the next block
        hand_store(hand + HAND_V + (li * 2 + (blk & 1)) * 128 + tid, __float_as_uint(v[li]));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
    } else {
      constexpr int NT_ = 256 - BN, VL = BN / 4, SL = BN / 16;   // storing threads; pieces per row of V and of S
      const int st = tid - BN;
      for (int s0 = 0; s0 < BM; s0 += U) {
        __syncthreads();
#pragma unroll
        for (int p0 = 0; p0 < U * VL; p0 += NT_) {
          const int p = p0 + st, row = s0 + p / VL, col = (p % VL) * 4;
          if (U * VL % NT_ == 0 || p < U * VL) {
            const u32x4 x = *(const u32x4 *)(lds + row * CP + col * 4);
            const int vo = t0 + row < a.T ? (((t0 + row) * a.B + b) * a.ld + n0 + col) * 4 : OOB;
            if (a.nt_store) __builtin_amdgcn_raw_buffer_store_b128(x, rV, vo, 0, NT);
            else __builtin_amdgcn_raw_buffer_store_b128(x, rV, vo, 0, 0);
          }
        }
#pragma unroll
        for (int p0 = 0; p0 < U * SL; p0 += NT_) {
          const int p = p0 + st, row = s0 + p / SL, col = (p % SL) * 16;
          if (p < U * SL) {
            u32x4 x;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const f32x4 f = *(const f32x4 *)(lds + row * CP + (col + 4 * q) * 4);
              x[q] = (f[0] > theta ? 1u : 0u) | (f[1] > theta ? 0x100u : 0u) | (f[2] > theta ? 0x10000u : 0u) |
                     (f[3] > theta ? 0x1000000u : 0u);
            }
            const int so = t0 + row < a.T ? ((t0 + row) * a.B + b) * a.ld + n0 + col : OOB;
            if (a.nt_store) __builtin_amdgcn_raw_buffer_store_b128(x, rS, so, 0, NT);
            else __builtin_amdgcn_raw_buffer_store_b128(x, rS, so, 0, 0);
          }
        }
        if (ROLE == 1 && (s0 + U) % 64 == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // a chunk's spikes are in the L2
      }
    }
    __syncthreads();
    if (ROLE == 1 && tid == 0) hand_store(hand + HAND_PAIR, hand_base + (t0 + BM) / 64);
    if (TS == 2 && blk + 1 < nblocks && tid == 0) hand_store(hand + li, hand_base + blk + 1);

    // 5. readout currents of the block: J^T (32 classes x 128 steps) = W_out^T S^T, a wavefront
    // takes 32 steps.  Second operand: lane -> step 32 wave + (lane & 31), neurons 16 kk + 8 h
    // .. +7, their spikes decided once more from V in the tile (exactly as in the scan) and
    // rounded to bfloat16 pairs.  The lane ends up with its step's currents, four consecutive
    // classes per register quad.
    if (READOUT && last) {
      f32x16 jt;
#pragma unroll
      for (int r = 0; r < 16; ++r) jt[r] = 0.f;
      const int row = 32 * wave + (lane & 31);          // (blocks of 64 steps: the first two wavefronts)
      if (row < BM) {
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const f32x4 p0 = *(const f32x4 *)(lds + row * CP + (16 * kk + 8 * h) * 4);
        const f32x4 p1 = *(const f32x4 *)(lds + row * CP + (16 * kk + 8 * h + 4) * 4);
        u32x4 sp;
        sp.x = (p0[0] > theta ? 0x3F80u : 0u) | (p0[1] > theta ? 0x3F800000u : 0u);
        sp.y = (p0[2] > theta ? 0x3F80u : 0u) | (p0[3] > theta ? 0x3F800000u : 0u);
        sp.z = (p1[0] > theta ? 0x3F80u : 0u) | (p1[1] > theta ? 0x3F800000u : 0u);
        sp.w = (p1[2] > theta ? 0x3F80u : 0u) | (p1[3] > theta ? 0x3F800000u : 0u);
        jt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[kk], __builtin_bit_cast(bf16x8, sp), jt, 0, 0, 0);
      }
      const rsrc_t rJ = make_rsrc(a.J, (unsigned)a.T * a.B * a.ldj * 4u);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = 8 * q + 4 * h;
        u32x4 x;
        x.x = __float_as_uint(jt[4 * q]); x.y = __float_as_uint(jt[4 * q + 1]);
        x.z = __float_as_uint(jt[4 * q + 2]); x.w = __float_as_uint(jt[4 * q + 3]);
        const int jo = t0 + row < a.T && c + 3 < a.ldj ? (((t0 + row) * a.B + b) * a.ldj + c) * 4 : OOB;
        __builtin_amdgcn_raw_buffer_store_b128(x, rJ, jo, 0, 0);
      }
      }
      if (LOSS) {
        // 6. readout scan of the block.  The LI readout is linear in its state, so the block's steps
        // are cut in eight segments of SEG: thread -> (segment tid / 32, class tid % 32).  A
        // segment is first integrated from a zero state, the results are exchanged, the state
        // entering each segment follows, and the segment is integrated again from it, step by
        // step as the sequential scan would (the scheme of readout_loss_kernel, which has the
        // eight wavefronts of a workgroup where this has the eight 32-lane groups).
        if (TS == 2 && blk > 0 && tid == 0) hand_wait(hand + 2, hand_base + blk, a.err);   // the readout has passed the block before
        __syncthreads();                              // V has been stored: the tile's space is free
        if (TS == 2 && blk > 0) {
          const uint32_t *src = hand + HAND_R + (((blk - 1) & 1) * 256 + tid) * 4;
          y_in = __uint_as_float(hand_load(src));
          best = __uint_as_float(hand_load(src + 1));
          tb = (int)hand_load(src + 2);
          ysum = __uint_as_float(hand_load(src + 3));
        }
        float *Jt = (float *)lds;
        if (row < BM) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f32x4 x = {jt[4 * q], jt[4 * q + 1], jt[4 * q + 2], jt[4 * q + 3]};
            *(f32x4 *)&Jt[row * JP + 8 * q + 4 * h] = x;
          }
        }
        __syncthreads();
        const int g = tid >> 5, c = tid & 31, ts0 = t0 + SEG * g;
        float j[SEG], e = 0.f;
#pragma unroll
        for (int k = 0; k < SEG; ++k) {
          j[k] = Jt[(SEG * g + k) * JP + c];
          e = beta_r * e + j[k];
        }
        x_e[par][g][c] = e;
        __syncthreads();
        float cst = y_in, y = 0.f;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
          if (v == g) y = cst;
          cst = bseg * cst + x_e[par][v][c];
        }
        y_in = cst;
#pragma unroll
        for (int k = 0; k < SEG; ++k) {
          y = beta_r * y + j[k];
          Jt[(SEG * g + k) * JP + c] = y;
          if (INTEGRAL) { if (ts0 + k < a.T) ysum += y; }
          else if (ts0 + k < a.T && y > best) { best = y; tb = ts0 + k; }
        }
        par ^= 1;
        if (TS == 2 && blk + 1 < nblocks) {           // hand the readout's state on
          uint32_t *dst = hand + HAND_R + ((blk & 1) * 256 + tid) * 4;
          hand_store(dst, __float_as_uint(y_in));
          hand_store(dst + 1, __float_as_uint(best));
          hand_store(dst + 2, (uint32_t)tb);
          hand_store(dst + 3, __float_as_uint(ysum));
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
        if (TS == 2 && blk + 1 < nblocks && tid == 0) hand_store(hand + 2, hand_base + blk + 1);
        const rsrc_t rY = make_rsrc(a.Y, (unsigned)a.T * a.B * a.ldj * 4u);
#pragma unroll
        for (int k = 0; k < BM / 32; ++k) {           // 8 lanes x 16 bytes per row, 32 rows per instruction
          const int r = 32 * k + (tid >> 3), cc = (tid & 7) * 4;
          const u32x4 x = *(const u32x4 *)&Jt[r * JP + cc];
          st_b128(rY, t0 + r < a.T && cc + 3 < a.ldj ? (((t0 + r) * a.B + b) * a.ldj + cc) * 4 : OOB, 0, x);
        }
      }
    }
    // A layer above reads the spikes of this block back from memory: they have reached the L2
    // (nothing of them is in this compute unit's L1) once the stores are acknowledged.
    if (!last) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                  // the next product's stages overwrite the tile
   });
  }

  if (LOSS && (TS == 1 || half == (nblocks - 1) % TS)) {   // (two workgroups per sample: the one of the last block)
    // first maximiser over the segments (integral loss: the sum of the segments' sums, in order)
    const int g = tid >> 5, c = tid & 31;
    x_best[g][c] = INTEGRAL ? ysum : best;
    x_tb[g][c] = tb;
    __syncthreads();
    best = x_best[0][c];
    tb = x_tb[0][c];
#pragma unroll
    for (int v = 1; v < 8; ++v) {
      const float bv = x_best[v][c];
      const int tv = x_tb[v][c];
      if (INTEGRAL) best += bv;
      else if (bv > best || (bv == best && tv < tb)) { best = bv; tb = tv; }
    }
    const bool live = c < a.C;
    const int p = b * a.ldj + c;
    if (live && g == 0) { a.z[p] = best; a.tstar[p] = tb; }
    // softmax cross-entropy of the sample (every 32-lane group, for dz)
    float m = live ? best : -INFINITY;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    const float ex = live ? expf(best - m) : 0.f;
    float sum = ex;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lab < 0 || lab >= a.C) { if (tid == 0) atomicOr(a.err, 1); lab = 0; }
    float zl = (live && c == lab) ? best : 0.f;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) zl += __shfl_xor(zl, o);
    const float d = live ? (ex / sum - (c == lab ? 1.f : 0.f)) / (float)a.B : 0.f;
    if (g == 0) {
      if (live) a.dz[p] = d;
      if (c == 0) a.loss_b[b] = m + logf(sum) - zl;
    }
    // dJ_t = h_t with h_t = beta h_{t+1} + dz [t == t*] (integral loss: dz at every step): entered
    // per segment in closed form, the recursion inside it
    const float l2b = log2f(beta_r);
    const rsrc_t rdJ = make_rsrc(a.dJ, (unsigned)a.T * a.B * a.ldj * 4u);
    uint32_t *Ht = (uint32_t *)lds;
    for (int t0 = 0; t0 < a.T; t0 += 128) {             // (128 steps at a time, whatever the block size above)
      const int ts0 = t0 + 16 * g;
      float hh;
      if (INTEGRAL) {
        const int n = a.T - (ts0 + 16);
        hh = n <= 0 ? 0.f : beta_r == 1.f ? d * (float)n : d * (1.f - exp2f((float)n * l2b)) / (1.f - beta_r);
      } else {
        const int n = tb - (ts0 + 16);
        hh = n > 0 ? d * exp2f((float)n * l2b) : n == 0 ? d : 0.f;
      }
      __syncthreads();                                // the previous block's rows have been stored
#pragma unroll
      for (int k = 15; k >= 0; --k) {
        hh = beta_r * hh + ((INTEGRAL ? ts0 + k < a.T : ts0 + k == tb) ? d : 0.f);
        Ht[(16 * g + k) * JP + c] = pack_hl(hh);
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int r = 32 * k + (tid >> 3), cc = (tid & 7) * 4;
        const u32x4 x = *(const u32x4 *)&Ht[r * JP + cc];
        st_b128(rdJ, t0 + r < a.T && cc + 3 < a.ldj ? (((t0 + r) * a.B + b) * a.ldj + cc) * 4 : OOB, 0, x);
      }
    }
  }
}

// LS = 2 (a pair of 128-neuron layers, NL = 2): the two layers of a sample run on two workgroups.
// The first takes the lower layer through the sample's blocks of 128 steps and, whenever the
// wavefronts that store V and S have another 64 steps acknowledged (the spikes are then in the L2
// the two workgroups share: ids 8 x parts apart run on the same XCD), raises a count in memory; the
// second takes the upper layer (and the readout) through blocks of 64 steps and waits for the count
// before each block's product, which reads those spikes.  The upper layer's product, scan and
// stores thereby run while the lower layer is still being scanned.  Only the second workgroup
// waits, and the first has the lower id, so it is never dispatched after the one waiting for it.
template <int TN, int NS = 3, int READOUT = 0, int NL = 1, bool PACKED = false, int TS = 1, int LS = 1>
__global__ __launch_bounds__(256, 2) void lif_layer_forward_kernel(const LayerForwardArgs a) {
  static_assert(!READOUT || TN == 2, "the readout variants hold the whole layer");
  static_assert(NL == 1 || (NL == 2 && TN == 2), "a chain of layers: whole layers of 128 neurons");
  static_assert(TS == 1 || (TS == 2 && TN == 2), "two workgroups per sample: whole layers of 128 neurons");
  static_assert(LS == 1 || (LS == 2 && NL == 2 && TS == 1), "a pair of layers on two workgroups");
  constexpr int TM = TS == 2 ? 1 : 2;                 // blocks of 64 steps when two workgroups share a sample's blocks
  typedef SpikeTile<2, 2, TM, TN, NS> Tile;
  constexpr int BN = Tile::BN, CP = BN * 4 + 16, TILE = Tile::BM * CP;
  constexpr int STAGES = Tile::lds_bytes(false) > Tile::lds_bytes(PACKED) ? Tile::lds_bytes(false) : Tile::lds_bytes(PACKED);
  constexpr int LDS_BYTES = STAGES > TILE ? STAGES : TILE;                 // the stages share the tile's space
  static_assert(LDS_BYTES <= 80 * 1024, "two workgroups per compute unit");
  __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
  __shared__ float x_e[2][8][32], x_best[8][32];
  __shared__ int x_tb[8][32];

  // Workgroup ids are dealt round-robin to the 8 XCDs: the parts of a sample take ids 8 apart.
  // The two workgroups of a sample part (TS = 2 or LS = 2) take ids 8 x parts apart, the one that
  // never waits for the other first.
  constexpr int WGS = TS * LS;
  const int parts = a.ld / BN;
  const int part = (blockIdx.x >> 3) % parts;
  const int half = WGS == 1 ? 0 : ((blockIdx.x >> 3) / parts) % WGS;
  const int b = (blockIdx.x >> 3) / (parts * WGS) * 8 + (blockIdx.x & 7);
  if (b >= a.B) return;
  if constexpr (LS == 2) {
    if (half == 0) lif_layer_forward_body<TN, NS, 0, 1, PACKED, 1, 2, 0, 1>(a, lds, x_e, x_best, x_tb, b, part, parts, 0);
    else lif_layer_forward_body<TN, NS, READOUT, 1, false, 1, 1, 1, 2>(a, lds, x_e, x_best, x_tb, b, part, parts, 0);
  } else {
    lif_layer_forward_body<TN, NS, READOUT, NL, PACKED, TS, TM, 0, 0>(a, lds, x_e, x_best, x_tb, b, part, parts, half);
  }
}

}  // namespace snn
