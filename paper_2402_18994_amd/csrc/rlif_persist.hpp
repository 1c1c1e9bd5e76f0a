// Forward time loop of a wide recurrent layer (Eq. 1-2 with the recurrent term: V_{t+1} = beta V_t + I_t +
// R s_t - theta s_t, s_{t+1} = [V_{t+1} > theta]) in ONE launch, on rounded weights.
//
// The per-step kernels (rlif.hpp) pay a launch and a pass of the weights through every compute unit
// per time step.  Here the grid of one workgroup per 32 neurons x 32 samples stays for all T steps:
//   * its 32 rows of R (up to 2048 columns of bfloat16, 128 KiB) are loaded into LDS once;
//   * V_t of its tile lives in registers;
//   * what a step needs from the other workgroups of its sample tile - the spikes of ALL neurons for
//     its 32 samples - is exchanged through memory as bits: every workgroup publishes one 64-bit word
//     per sample, {the spikes of its 32 neurons, the step they belong to}, and reads ld / 32 words per
//     sample.  The words are written and read with relaxed device-scope 8-byte accesses (single-copy
//     atomic; they bypass the caches that are not shared by all compute units), so a word is its own
//     flag: a reader loads the words it needs until each carries the step it waits for.  Nothing else
//     orders the workgroups: one propagation of a store and one load round trip per step.  Two word
//     buffers by parity of t: a workgroup overwrites its word of step t only after it has read every
//     word of step t + 1, which their writers published after reading step t.
//     (A first version with 4-byte words and a counter per sample tile, raised after the stores were
//     acknowledged and polled before the words were read, took 13 us per step: three round trips.)
// Every workgroup must be resident at once: the launch is refused unless the grid fits the compute
// units at one workgroup each (the LDS use enforces one per unit).  A wait polls at most 2^18 times
// (about a second; SNN_OPT_WAIT_LIMIT_LOG2); on a time-out the workgroup sets bit 1 of the error word and a flag that ends all
// waiting in every workgroup, so the grid always drains and the host reports the failure.
//
// The arithmetic is that of rlif_step_forward_kernel in the same order (a wavefront walks the same
// quarter of the contraction in the same steps, the four partial sums are added in the same order):
// the results are bit-identical.
#pragma once
#include "layer_forward.hpp"
#include "rlif.hpp"

namespace snn {

struct RlifPersist {
  static constexpr int MAXK = 2048;                    // widest layer (contraction length, padded)
  static constexpr int PITCH = MAXK * 2 + 16;          // bytes between rows of the slab: 16-byte reads of 16 rows spread over all banks
  static constexpr int SBP = MAXK / 8 + 4;             // bytes between the samples' bit rows in LDS
  static constexpr int LDS_BYTES = 32 * PITCH + 4 * 16 * 64 * 4 + 32 * SBP + 32 * 4;
  static constexpr int WPT = MAXK / 32 * 32 / 256;     // words a thread fetches per step (at most)
};

// words [2][SB * 32][ldqr / 32] and the abort flag are zero at the launch (S_0 = 0 is what buffer 0 then says).
// max_polls: bound of a wait; tag_bias: 0, or (tests of the time-out path) a value that makes every wait
// expect a step nobody publishes.
__global__ __launch_bounds__(256) void rlif_persist_forward_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                                   uint8_t *__restrict__ S, const uint16_t *__restrict__ QRf,
                                                                   int ldqr, int T, int B, int ld, const float *__restrict__ beta_v,
                                                                   float theta, uint64_t *words, uint32_t *abort_flag, int *err, int max_polls,
                                                                   uint32_t tag_bias) {
  typedef RlifPersist G;
  __shared__ __attribute__((aligned(16))) char lds[G::LDS_BYTES];
  char *const slab = lds;
  float(*const red)[16][64] = (float(*)[16][64])(lds + 32 * G::PITCH);
  uint8_t *const sb = (uint8_t *)(lds + 32 * G::PITCH + 4 * 16 * 64 * 4);
  uint32_t *const pk = (uint32_t *)(sb + 32 * G::SBP);

  const int SB = gridDim.y, NT = gridDim.x;            // sample tiles, neuron tiles (= workgroups per sample tile)
  const int nt = blockIdx.x, st = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, h = lane >> 5;
  const int KW = ldqr >> 5;                            // dwords of a sample's bit row
  const size_t stride = (size_t)B * ld;

  // the slab: row r of the tile at r * PITCH
  for (int r = 0; r < 32; ++r)
    for (int u = tid; u < ldqr / 8; u += 256)
      *(u32x4 *)(slab + r * G::PITCH + 16 * u) = *(const u32x4 *)(QRf + (size_t)(nt * 32 + r) * ldqr + 8 * u);

  const int b = st * 32 + (lane & 31);
  const int n = nt * 32 + 8 * w + 4 * h;
  const bool upd = b < B && n < ld;
  const size_t o = upd ? (size_t)b * ld + n : 0;
  const float4 be = *(const float4 *)(beta_v + (upd ? n : 0));
  const float b4[4] = {be.x, be.y, be.z, be.w};
  float v4[4] = {0.f, 0.f, 0.f, 0.f};                  // V_0 = 0
  uint32_t sp = 0;                                     // S_0 = 0 (one bit per neuron of the thread)
  bool aborted = false;                                // a wait timed out somewhere: no more waiting
  if (upd) {
    *(float4 *)(V + o) = make_float4(0.f, 0.f, 0.f, 0.f);
    *(uint32_t *)(S + o) = 0u;
  }
  for (int i = tid; i < 32 * G::SBP / 4; i += 256) ((uint32_t *)sb)[i] = 0u;   // (bits beyond the publishers' words stay zero)
  const int steps = ldqr >> 6;                         // MFMA steps (16 k) of a wavefront: a quarter of the contraction
  const char *const fa = slab + (lane & 31) * G::PITCH + (w * (ldqr >> 2) + 8 * h) * 2;
  const uint8_t *const fb = sb + (lane & 31) * G::SBP + w * (ldqr >> 5) + h;
  __syncthreads();

  for (int t = 0; t + 1 < T; ++t) {
    // operands of the update do not depend on the product: ask for them first
    const float4 cur = upd ? *(const float4 *)(I + t * stride + o) : make_float4(0.f, 0.f, 0.f, 0.f);
    if (tid < 32) pk[tid] = 0u;                        // (two barriers lie between this and the first atomicOr)
    // the bits of s_t from every workgroup of the sample tile: each thread fetches its words until they
    // carry step t
    {
      const uint64_t *src = words + ((size_t)(t & 1) * SB + st) * 32 * KW;
      const uint32_t want = (uint32_t)t + (t ? tag_bias : 0u);
      uint64_t x[G::WPT] = {};
      int at[G::WPT];                                    // word of sample i / NT, publisher i % NT (words beyond the publishers stay zero)
#pragma unroll
      for (int j = 0; j < G::WPT; ++j) {
        const int i = tid + 256 * j, smp = i / NT;
        at[j] = i < 32 * NT ? smp * KW + (i - smp * NT) : -1;
      }
      bool ok = aborted;
      for (int spins = 0; !ok; ++spins) {
        ok = true;
#pragma unroll
        for (int j = 0; j < G::WPT; ++j)
          if (at[j] >= 0 && (spins == 0 || (uint32_t)(x[j] >> 32) != want))
            x[j] = __hip_atomic_load(src + at[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int j = 0; j < G::WPT; ++j)
          if (at[j] >= 0 && (uint32_t)(x[j] >> 32) != want) ok = false;
        if (!ok) {
          if ((spins & 15) == 15 && hand_load(abort_flag)) aborted = true;
          if (spins >= max_polls) { atomicOr(err, 2); hand_store(abort_flag, 1u); aborted = true; }
          if (aborted) break;
          __builtin_amdgcn_s_sleep(1);
        }
      }
#pragma unroll
      for (int j = 0; j < G::WPT; ++j)
        if (at[j] >= 0) *(uint32_t *)(sb + 4 * at[j] + (at[j] / KW) * (G::SBP - 4 * KW)) = aborted ? 0u : (uint32_t)x[j];
    }
    __syncthreads();
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    // Four steps at a time, the fragments of the next four asked for before these are multiplied (left
    // as a plain loop, every step waited a whole LDS round trip: 157 cycles per MFMA).  Eight spikes of
    // the lane's sample are the bits of one byte, bit r = neuron 8 (..) + r: z holds the byte at bits
    // 0..7 and again at bits 15..22; shifted left by 14 - 2 j, bit 14 is element 2 j and bit 30 element
    // 2 j + 1, i.e. the bfloat16 pair 2.0 x spikes (the sums are halved below: exact).
    bf16x8 wf[2][4];
    uint32_t sv[2][4];
    auto fetch = [&](int g, int s0) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        wf[g][q] = *(const bf16x8 *)(fa + 32 * (s0 + q));
        sv[g][q] = fb[2 * (s0 + q)];
      }
    };
    auto multiply = [&](int g) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t z = sv[g][q] | (sv[g][q] << 15);
        u32x4 d;
        d.x = (z << 14) & 0x40004000u;
        d.y = (z << 12) & 0x40004000u;
        d.z = (z << 10) & 0x40004000u;
        d.w = (z << 8) & 0x40004000u;
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[g][q], __builtin_bit_cast(bf16x8, d), acc, 0, 0, 0);
      }
    };
    // (branch-free body: with a fetch or a multiply under a condition the compiler moved the accumulator
    // between its two register files in every iteration, draining the MFMA chain each time)
    fetch(0, 0);
    for (int s = 0; s < steps; s += 4) {                 // (steps is a multiple of 4)
      fetch(1, min(s + 4, steps - 4));
      multiply(0);
#pragma unroll
      for (int q = 0; q < 4; ++q) { wf[0][q] = wf[1][q]; sv[0][q] = sv[1][q]; }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] *= 0.5f;
    const f32x4 sum = rlif_reduce(acc, red, w, lane);
    const float c4[4] = {cur.x, cur.y, cur.z, cur.w};
    uint32_t out = 0, nib = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float s = (float)((sp >> i) & 1u);
      v4[i] = b4[i] * v4[i] + c4[i] + sum[i] - theta * s;
      const uint32_t f = upd && v4[i] > theta ? 1u : 0u;
      nib |= f << i;
      out |= f << (8 * i);
    }
    sp = nib;
    if (nib) atomicOr(&pk[lane & 31], nib << (8 * w + 4 * h));
    __syncthreads();
    // publish s_{t+1}: one word per sample
    if (tid < 32)
      __hip_atomic_store(words + (((size_t)((t + 1) & 1) * SB + st) * 32 + tid) * KW + nt,
                         (uint64_t)pk[tid] | ((uint64_t)(uint32_t)(t + 1) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (upd) {
      *(float4 *)(V + (t + 1) * stride + o) = make_float4(v4[0], v4[1], v4[2], v4[3]);
      *(uint32_t *)(S + (t + 1) * stride + o) = out;
    }
  }
}

// Bytes of the exchange space: two word buffers and the abort flag (a multiple of 256).
static size_t rlif_persist_bytes(int B, int ldqr) {
  const size_t sb = (size_t)(B + 31) / 32;
  return (2 * sb * 32 * (size_t)(ldqr / 32) * 8 + 8 + 255) / 256 * 256;
}

// Whether the layer's forward loop can run as one launch on `cus` compute units.
static bool rlif_persist_fits(int B, int ld, int ldqr, int cus) {
  return ld > 128 && ldqr % 256 == 0 && ldqr <= RlifPersist::MAXK && ld <= ldqr && ((ld + 31) / 32) * ((B + 31) / 32) <= cus;
}

static hipError_t rlif_persist_forward(hipStream_t st, int T, int B, int ld, const float *I, float *V, uint8_t *S,
                                       const uint16_t *QRf, int ldqr, const float *beta, float theta, void *space, int *err,
                                       int max_polls, bool fault) {
  const int sb = (B + 31) / 32;
  hipError_t e = fill_zero(st, space, rlif_persist_bytes(B, ldqr));
  if (e != hipSuccess) return e;
  uint64_t *words = (uint64_t *)space;
  uint32_t *abort_flag = (uint32_t *)(words + 2 * (size_t)sb * 32 * (ldqr / 32));
  hipLaunchKernelGGL(rlif_persist_forward_kernel, dim3((ld + 31) / 32, sb), dim3(256), 0, st, I, V, S, QRf, ldqr, T, B, ld, beta,
                     theta, words, abort_flag, err, max_polls, fault ? 0x40000000u : 0u);
  return hipGetLastError();
}

}  // namespace snn
