// Recurrent LIF layers: V_{t+1} = beta V_t + I_t + S_t R - theta S_t, with S_t the spikes
// just emitted from V_t (R is [from][to]).  Every step needs all N spikes of a sample from
// the step before.  Layers of up to 128 neurons run their whole time loop in one kernel (a
// workgroup owns a batch tile and all neurons).  Wider layers walk time on the host side of
// the stream: one launch per step, each a [B x N] x [N x N] MFMA product whose epilogue
// applies the LIF update (forward) or the surrogate-gradient recursion (reverse); stream
// order is the inter-step barrier.
#pragma once
#include "gemm.hpp"
#include "scan.hpp"

namespace snn {

static hipError_t fill_zero(hipStream_t st, void *p, size_t bytes) {
  const long long n = (long long)(bytes / 4);
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint32_t *)p, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------- narrow layers: one launch
// For N <= 128 a workgroup can own a batch tile of 32 samples with ALL neurons of the layer:
// the recurrence then never leaves the workgroup and the whole time loop runs inside one
// kernel.  The product is taken transposed, (S_t R)^T = R^T S_t^T: the MFMA's row operand is a
// 32-neuron slab of R^T (or of R for the reverse pass), loaded once and kept in registers for
// all T steps; the column operand is the 32 x 128 tile of the samples' current spikes (or of
// the planes of g), exchanged between the four wavefronts through LDS, double-buffered, one
// barrier per step.  In the 32x32 accumulator a lane holds sample (lane & 31) and sixteen
// neurons in four groups of four adjacent ones, so state, loads and stores are per-lane
// 16-byte vectors and the LIF update needs no shuffles.  Wavefront w owns neurons
// [32w, 32w+32).  Rows of I (or dS and V) are fetched PF steps ahead of their use.
// These 32-sample kernels are followed by the ones in use by default, which tile the batch by
// 16 samples (16x16x32 MFMAs, eight wavefronts of 16 neurons): the step is a dependent chain -
// spikes or planes of g into LDS, barrier, fragments, products, update - and its length is the
// number of values a lane carries: 16 here, 4 there (0.97 -> 0.43 us per forward step,
// 1.64 -> 0.64 per reverse step at 128 neurons).
constexpr int RL_PITCH = 272;                 // bytes per sample row of an exchange tile (128 bf16 + pad)

// The sixteen-byte fragment of a weight plane [row][k] (k contiguous, pitch ldq) for MFMA step ks.
__device__ __forceinline__ bf16x8 rl_weight_frag(rsrc_t r, int row, int ldq, int ks, int lane) {
  const int k = 16 * ks + 8 * (lane >> 5);
  const u32x4 v = ld_b128(r, k < ldq ? (row * ldq + k) * 2 : OOB, 0);
  return __builtin_bit_cast(bf16x8, v);
}

// Row pitches of the LDS stage through which the 16-sample kernel below stores V_t and S_t as
// whole rows.  (This 32-sample kernel stores straight from the accumulator layout, 32 sample rows
// of 32 bytes per instruction, and serves rows that are no multiple of 16 neurons.)
constexpr int RL_VP = 132;                    // floats per sample row of the V stage (128 + pad)
constexpr int RL_SP = 144;                    // bytes per sample row of the S stage (128 + pad)
template <int NP>   // NP weight planes: 1 (bfloat16 weights) or 3 (fp32 as hi + mid + lo)
__global__ __launch_bounds__(256) void rlif_forward_fused_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                                 uint8_t *__restrict__ S,
                                                                 const uint16_t *__restrict__ QRf, int ldqr,
                                                                 long long qr_plane, int T, int B, int N, int ld,
                                                                 const float *__restrict__ beta_v, float theta) {
  constexpr int PF = 4;
  __shared__ __align__(16) char xs[2][32 * RL_PITCH];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = blockIdx.x * 32 + (lane & 31);
  const int row4 = B * ld * 4;
  const unsigned bytes = (unsigned)T * B * ld * 4u;
  const rsrc_t rI = make_rsrc(I, bytes), rV = make_rsrc(V, bytes), rS = make_rsrc(S, bytes / 4);
  const rsrc_t rQ = make_rsrc(QRf, (unsigned)(NP * qr_plane * 2));

  bf16x8 wf[NP][8];                             // R^T[32w + (lane&31)][:], all planes, all k steps
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      wf[p][ks] = rl_weight_frag(rQ, (int)(p * (qr_plane / ldqr)) + 32 * w + (lane & 31), ldqr, ks, lane);

  int vo4[4], vo1[4], xo[4];                    // per group of four neurons
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int n = 32 * w + 8 * g + 4 * (lane >> 5);
    const bool ok = b < B && n < ld;
    vo4[g] = ok ? (b * ld + n) * 4 : OOB;
    vo1[g] = ok ? b * ld + n : OOB;
    xo[g] = (lane & 31) * RL_PITCH + n * 2;
  }
  float v[16], beta[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    v[i] = 0.f;                                  // V_0 = 0
    const int n = 32 * w + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
    beta[i] = n < ld ? beta_v[n] : 0.f;          // one decay per neuron
  }
  u32x4 cur[PF][4];
#pragma unroll
  for (int d = 0; d < PF; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g) cur[d][g] = ld_b128(rI, vo4[g], min(d, T - 1) * row4);

  // One step.  The chain that bounds it is serial - spikes into LDS, barrier, fragment reads, the
  // MFMAs, the state update - so everything that does not depend on the product is issued
  // while the MFMAs run: the stores of V_t and S_t sit between the MFMAs and the update, and
  // the eight products of a step go to two accumulators (even and odd k steps) so that only
  // four of them depend on each other.
  auto step = [&](u32x4 (&in)[4], int t) {
    uint32_t sp[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) sp[i] = v[i] > theta ? 1u : 0u;
    char *x = xs[t & 1];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x2 sx;                                  // four spikes as bfloat16 0.0 / 1.0
      sx[0] = (sp[4 * g] | (sp[4 * g + 1] << 16)) * 0x3F80u;
      sx[1] = (sp[4 * g + 2] | (sp[4 * g + 3] << 16)) * 0x3F80u;
      *(u32x2 *)(x + xo[g]) = sx;
    }
    f32x16 acc, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = acc1[r] = 0.f;
    lds_barrier();
    if (t + 1 < T) {                             // the last state is not used
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 sf = *(const bf16x8 *)(x + (lane & 31) * RL_PITCH + (16 * ks + 8 * (lane >> 5)) * 2);
#pragma unroll
        for (int p = NP - 1; p >= 0; --p) {
          if (ks & 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[p][ks], sf, acc1, 0, 0, 0);
          else acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[p][ks], sf, acc, 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x4 vv;
#pragma unroll
      for (int i = 0; i < 4; ++i) vv[i] = __float_as_uint(v[4 * g + i]);
      st_b128(rV, vo4[g], t * row4, vv);
      st_b32(rS, vo1[g], t * (row4 >> 2), sp[4 * g] | (sp[4 * g + 1] << 8) | (sp[4 * g + 2] << 16) | (sp[4 * g + 3] << 24));
    }
    // accumulator register r: neuron 32w + 8*(r/4) + 4*(lane/32) + r%4, i.e. group r/4, element r%4
#pragma unroll
    for (int i = 0; i < 16; ++i)
      v[i] = beta[i] * v[i] + __uint_as_float(in[i >> 2][i & 3]) + (acc[i] + acc1[i]) - (sp[i] ? theta : 0.f);
#pragma unroll
    for (int g = 0; g < 4; ++g) in[g] = ld_b128(rI, vo4[g], min(t + PF, T - 1) * row4);
  };
  int t = 0;
  for (; t + PF <= T; t += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) step(cur[d], t + d);
  }
#pragma unroll
  for (int d = 0; d < PF; ++d)
    if (t + d < T) step(cur[d], t + d);
}

// The same forward pass on tiles of 16 samples (16x16x32 MFMAs): a lane then carries 8 neurons
// of one sample instead of 16 - half the compares, packs, updates, loads and LDS traffic in the
// step's dependent chain - and a batch fills twice as many compute units.  Wavefront w still
// owns neurons [32w, 32w+32), as two row tiles of 16; in a tile's accumulator the lane holds
// sample (lane & 15) and the four adjacent neurons 4 (lane / 16) .. +3.  Rows of a multiple of 16
// neurons only: V_t and S_t always leave through the LDS stage (rows 2 (NWV k + w) + lane/32 of
// the tile for V instruction k; the first two wavefronts store S, rows 8w + lane/8).
// NTW: row tiles per wavefront.  2: four wavefronts; 1: eight wavefronts of 16 neurons each, a
// lane then carries 4 neurons (half the dependent chain again, two wavefronts per SIMD).
template <int NP, int NTW>
__global__ __launch_bounds__(512 / NTW) void rlif_forward_fused16_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                                   uint8_t *__restrict__ S,
                                                                   const uint16_t *__restrict__ QRf, int ldqr,
                                                                   long long qr_plane, int T, int B, int N, int ld,
                                                                   const float *__restrict__ beta_v, float theta) {
  constexpr int PF = 8;                         // steps of I in flight (8: 108 us for the two layers of 700-128-128-20, 4: 111)
  __shared__ __align__(16) char xs[2][16 * RL_PITCH];
  __shared__ __align__(16) float vstage[2][16 * RL_VP];
  __shared__ __align__(16) uint8_t sstage[2][16 * RL_SP];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int bl = lane & 15, q = lane >> 4;       // sample of the tile, group of four neurons / of eight k
  const int b = blockIdx.x * 16 + bl;
  const int row4 = B * ld * 4;
  const unsigned bytes = (unsigned)T * B * ld * 4u;
  const rsrc_t rI = make_rsrc(I, bytes), rV = make_rsrc(V, bytes), rS = make_rsrc(S, bytes / 4);
  const rsrc_t rQ = make_rsrc(QRf, (unsigned)(NP * qr_plane * 2));

  // R^T[16 (NTW w + i) + (lane & 15)][32 ks + 8 q .. +7], all planes: resident
  constexpr int NWV = 8 / NTW;                   // wavefronts
  bf16x8 wf[NP][NTW][4];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int i = 0; i < NTW; ++i)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int row = (int)(p * (qr_plane / ldqr)) + 16 * (NTW * w + i) + bl, k = 32 * ks + 8 * q;
        wf[p][i][ks] = __builtin_bit_cast(bf16x8, ld_b128(rQ, k < ldqr ? (row * ldqr + k) * 2 : OOB, 0));
      }

  int vo4[NTW], xo[NTW], nn[NTW];
#pragma unroll
  for (int i = 0; i < NTW; ++i) {
    nn[i] = 16 * (NTW * w + i) + 4 * q;
    vo4[i] = b < B && nn[i] < ld ? (b * ld + nn[i]) * 4 : OOB;
    xo[i] = bl * RL_PITCH + nn[i] * 2;
  }
  int vro[NTW], vlo[NTW], sro, slo;
#pragma unroll
  for (int k = 0; k < NTW; ++k) {
    const int r = 2 * (NWV * k + w) + (lane >> 5), c = (lane & 31) * 4, bb = blockIdx.x * 16 + r;
    vro[k] = bb < B && c < ld ? (bb * ld + c) * 4 : OOB;
    vlo[k] = r * RL_VP + c;
  }
  {
    const int r = 8 * (w & 1) + (lane >> 3), c = (lane & 7) * 16, bb = blockIdx.x * 16 + r;
    sro = w < 2 && bb < B && c < ld ? bb * ld + c : OOB;
    slo = r * RL_SP + c;
  }
  float v[4 * NTW], beta[4 * NTW];
#pragma unroll
  for (int e = 0; e < 4 * NTW; ++e) {
    v[e] = 0.f;                                  // V_0 = 0
    const int n = nn[e >> 2] + (e & 3);
    beta[e] = n < ld ? beta_v[n] : 0.f;
  }
  u32x4 cur[PF][NTW];
#pragma unroll
  for (int d = 0; d < PF; ++d)
#pragma unroll
    for (int i = 0; i < NTW; ++i) cur[d][i] = ld_b128(rI, vo4[i], min(d, T - 1) * row4);

  auto step = [&](u32x4 (&in)[NTW], int t) {
    uint32_t sp[4 * NTW];
#pragma unroll
    for (int e = 0; e < 4 * NTW; ++e) sp[e] = v[e] > theta ? 1u : 0u;
    char *x = xs[t & 1];
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
      u32x2 sx;                                  // four spikes as bfloat16 0.0 / 1.0
      sx[0] = (sp[4 * i] | (sp[4 * i + 1] << 16)) * 0x3F80u;
      sx[1] = (sp[4 * i + 2] | (sp[4 * i + 3] << 16)) * 0x3F80u;
      *(u32x2 *)(x + xo[i]) = sx;
      f32x4 vv = {v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]};
      *(f32x4 *)&vstage[t & 1][bl * RL_VP + nn[i]] = vv;
      *(uint32_t *)&sstage[t & 1][bl * RL_SP + nn[i]] =
          sp[4 * i] | (sp[4 * i + 1] << 8) | (sp[4 * i + 2] << 16) | (sp[4 * i + 3] << 24);
    }
    f32x4 acc[NTW][2];                             // [tile][even / odd k step]
#pragma unroll
    for (int i = 0; i < NTW; ++i)
#pragma unroll
      for (int o = 0; o < 2; ++o) acc[i][o] = f32x4{0.f, 0.f, 0.f, 0.f};
    lds_barrier();
    if (t + 1 < T) {                             // the last state is not used
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 sf = *(const bf16x8 *)(x + bl * RL_PITCH + (32 * ks + 8 * q) * 2);
#pragma unroll
        for (int p = NP - 1; p >= 0; --p)
#pragma unroll
          for (int i = 0; i < NTW; ++i)
            acc[i][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[p][i][ks], sf, acc[i][ks & 1], 0, 0, 0);
      }
    }
#pragma unroll
    for (int k = 0; k < NTW; ++k) st_b128(rV, vro[k], t * row4, *(const u32x4 *)&vstage[t & 1][vlo[k]]);
    st_b128(rS, sro, t * (row4 >> 2), *(const u32x4 *)&sstage[t & 1][slo]);
#pragma unroll
    for (int e = 0; e < 4 * NTW; ++e)
      v[e] = beta[e] * v[e] + __uint_as_float(in[e >> 2][e & 3]) + (acc[e >> 2][0][e & 3] + acc[e >> 2][1][e & 3]) -
             (sp[e] ? theta : 0.f);
#pragma unroll
    for (int i = 0; i < NTW; ++i) in[i] = ld_b128(rI, vo4[i], min(t + PF, T - 1) * row4);
  };
  int t = 0;
  for (; t + PF <= T; t += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) step(cur[d], t + d);
  }
#pragma unroll
  for (int d = 0; d < PF; ++d)
    if (t + d < T) step(cur[d], t + d);
}

// Reverse pass of these layers: g <- beta g + surr(V_t - theta) (dS_t - theta g + g R^T), dI_t = g
// before the update.  g is real-valued, so it enters the product as bfloat16 planes (hi + lo
// with bfloat16 weights, hi + mid + lo with fp32 weights); (g R^T)^T = R g^T with R[from][to]
// as the row operand.
// The reverse pass on tiles of 16 samples, as rlif_forward_fused16_kernel: a lane carries 8
// neurons of one sample, wavefront w two row tiles of 16 neurons of R (NTW = 2), or 4 and one
// on eight wavefronts (NTW = 1).
template <int NP, int SURR, int NTW>
__global__ __launch_bounds__(512 / NTW) void rlif_reverse_fused16_kernel(const float *__restrict__ dS,
                                                                   const float *__restrict__ V,
                                                                   uint32_t *__restrict__ dI,
                                                                   const uint16_t *__restrict__ QRb, int ldqr,
                                                                   long long qr_plane, int T, int B, int N, int ld,
                                                                   const float *__restrict__ beta_v, float theta, float slope,
                                                                   float *__restrict__ db_part) {
  constexpr int PF = 3;                         // steps of dS and V in flight (3: 154 us for the two layers of 700-128-128-20, 2: 166, 4: 178)
  constexpr int GP = NP == 1 ? 2 : 3;           // planes of g
  constexpr bool HL = NP == 1;                  // dI is stored in hi/lo form with bfloat16 weights
  __shared__ __align__(16) char xs[2][GP][16 * RL_PITCH];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int bl = lane & 15, q4 = lane >> 4;
  const int b = blockIdx.x * 16 + bl;
  const int row4 = B * ld * 4;
  const unsigned bytes = (unsigned)T * B * ld * 4u;
  const rsrc_t rdS = make_rsrc(dS, bytes), rV = make_rsrc(V, bytes), rdI = make_rsrc(dI, bytes);
  const rsrc_t rQ = make_rsrc(QRb, (unsigned)(NP * qr_plane * 2));

  bf16x8 wf[NP][NTW][4];                        // R[16 (NTW w + i) + (lane & 15)][32 ks + 8 (lane / 16) .. +7]
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int i = 0; i < NTW; ++i)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int row = (int)(p * (qr_plane / ldqr)) + 16 * (NTW * w + i) + bl, k = 32 * ks + 8 * q4;
        wf[p][i][ks] = __builtin_bit_cast(bf16x8, ld_b128(rQ, k < ldqr ? (row * ldqr + k) * 2 : OOB, 0));
      }

  int vo4[NTW], xo[NTW], nn[NTW];
#pragma unroll
  for (int i = 0; i < NTW; ++i) {
    nn[i] = 16 * (NTW * w + i) + 4 * q4;
    vo4[i] = b < B && nn[i] < ld ? (b * ld + nn[i]) * 4 : OOB;
    xo[i] = bl * RL_PITCH + nn[i] * 2;
  }
  float gv[4 * NTW], beta[4 * NTW], db[4 * NTW];
#pragma unroll
  for (int e = 0; e < 4 * NTW; ++e) {
    gv[e] = 0.f;                                 // g_T = 0
    db[e] = 0.f;                                 // sum over t of g_{t+1} V_t
    const int n = nn[e >> 2] + (e & 3);
    beta[e] = n < ld ? beta_v[n] : 0.f;
  }
  u32x4 cds[PF][NTW], cv[PF][NTW];
#pragma unroll
  for (int d = 0; d < PF; ++d)
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
      const int so = max(T - 1 - d, 0) * row4;
      cds[d][i] = ld_b128(rdS, vo4[i], so);
      cv[d][i] = ld_b128(rV, vo4[i], so);
    }

  auto step = [&](u32x4 (&ds)[NTW], u32x4 (&vv)[NTW], int t) {
    char *x = (char *)xs[t & 1];
    u32x4 o[NTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
      uint32_t pl[GP][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float gg = gv[4 * i + j];
        if (HL) {
          const uint32_t hl = pack_hl(gg);
          o[i][j] = hl;
          pl[0][j] = hl & 0xFFFFu;
          pl[1][j] = hl >> 16;
        } else {
          o[i][j] = __float_as_uint(gg);
#pragma unroll
          for (int q = 0; q < GP; ++q) pl[q][j] = bf16_piece(gg, q);
        }
      }
#pragma unroll
      for (int q = 0; q < GP; ++q) {
        u32x2 px;
        px[0] = pl[q][0] | (pl[q][1] << 16);
        px[1] = pl[q][2] | (pl[q][3] << 16);
        *(u32x2 *)(x + q * 16 * RL_PITCH + xo[i]) = px;
      }
    }
    f32x4 acc[NTW][2];                             // [tile][even / odd k step]
#pragma unroll
    for (int i = 0; i < NTW; ++i)
#pragma unroll
      for (int o2 = 0; o2 < 2; ++o2) acc[i][o2] = f32x4{0.f, 0.f, 0.f, 0.f};
    lds_barrier();
    if (t > 0) {                                 // the g leaving step 0 is not used
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8 gf[GP];
#pragma unroll
        for (int q = 0; q < GP; ++q)
          gf[q] = *(const bf16x8 *)(x + q * 16 * RL_PITCH + bl * RL_PITCH + (32 * ks + 8 * q4) * 2);
        // smallest products first
#pragma unroll
        for (int sum = NP + GP - 2; sum >= 0; --sum)
#pragma unroll
          for (int p = 0; p < NP; ++p) {
            const int q = sum - p;
            if (q >= 0 && q < GP && (NP == 1 || p + q < 3)) {
#pragma unroll
              for (int i = 0; i < NTW; ++i)
                acc[i][ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[p][i][ks], gf[q], acc[i][ks & 1], 0, 0, 0);
            }
          }
      }
    }
#pragma unroll
    for (int i = 0; i < NTW; ++i) st_b128(rdI, vo4[i], t * row4, o[i]);
    float sg[4 * NTW];
#pragma unroll
    for (int e = 0; e < 4 * NTW; ++e) sg[e] = surr_rcp<SURR>(slope, __uint_as_float(vv[e >> 2][e & 3]) - theta);
#pragma unroll
    for (int e = 0; e < 4 * NTW; ++e) {
      const float qq = __uint_as_float(ds[e >> 2][e & 3]) - theta * gv[e] + (acc[e >> 2][0][e & 3] + acc[e >> 2][1][e & 3]);
      const float vt = __uint_as_float(vv[e >> 2][e & 3]);
      db[e] += gv[e] * vt;
      gv[e] = beta[e] * gv[e] + sg[e] * qq;
    }
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
      const int so = max(t - PF, 0) * row4;
      ds[i] = ld_b128(rdS, vo4[i], so);
      vv[i] = ld_b128(rV, vo4[i], so);
    }
  };
  int t = T - 1;
  for (; t - PF + 1 >= 0; t -= PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) step(cds[d], cv[d], t - d);
  }
#pragma unroll
  for (int d = 0; d < PF; ++d)
    if (t - d >= 0) step(cds[d], cv[d], t - d);
  if (db_part) {                                 // per sample; summed over the batch by the reduction launch
#pragma unroll
    for (int i = 0; i < NTW; ++i)
      if (b < B && nn[i] < ld)
        *(float4 *)(db_part + (size_t)b * ld + nn[i]) = make_float4(db[4 * i], db[4 * i + 1], db[4 * i + 2], db[4 * i + 3]);
  }
}

// ---------------------------------------------------------------- wide layers: one launch per step
// Wider layers do not fit a workgroup, so time is walked on the host side of the stream and
// stream order is the inter-step barrier.  One step is the transposed product of the fused
// kernels above, tiled 32 neurons x 32 samples per workgroup; the four wavefronts split the
// contraction and add their accumulators through LDS, after which wavefront w applies the
// LIF update (or the surrogate recursion) to neuron group w of the tile.  Each wavefront
// walks its share of the contraction in 64-wide tiles of its own: rows are fetched with
// 16-byte loads that cover whole cache lines (a fragment-shaped load would touch 32 lines per
// instruction and leave the kernel bound by address processing), converted, written to a
// wavefront-private LDS tile in the swizzled layout of the product kernels and read back as
// MFMA fragments; no workgroup barrier is needed until the final sum.  Neuron tiles are dealt
// to XCDs so that XCD x only ever reads the rows x, x+8, .. (in units of 32) of the weight
// matrix.
struct RlifStepMap {
  int nt, st;          // neuron tile, sample tile
  bool live;
};
__device__ __forceinline__ RlifStepMap rlif_step_map(int n_tiles, int s_tiles) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  RlifStepMap m;
  m.st = slot % s_tiles;
  m.nt = (slot / s_tiles) * 8 + xcd;
  m.live = m.nt < n_tiles;
  return m;
}
static inline unsigned rlif_step_grid(int N, int B) {
  const int n_tiles = (N + 31) / 32, s_tiles = (B + 31) / 32;
  return 8u * s_tiles * ((n_tiles + 7) / 8);
}

// Sums the four wavefronts' accumulators; returns registers 4w..4w+3 (neuron group w).
__device__ __forceinline__ f32x4 rlif_reduce(const f32x16 &acc, float (*red)[16][64], int w, int lane) {
#pragma unroll
  for (int r = 0; r < 16; ++r) red[w][r][lane] = acc[r];
  __syncthreads();
  f32x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (red[0][4 * w + i][lane] + red[1][4 * w + i][lane]) + (red[2][4 * w + i][lane] + red[3][4 * w + i][lane]);
  return o;
}

// Weight tile of a wavefront: 32 rows x 64 contraction elements of every plane, four
// 16-byte loads per plane (lane: row lane/8 + 8j, chunk lane%8).
template <int NP> struct RlifWeightTile {
  u32x4 r[NP][4];
  __device__ __forceinline__ void load(rsrc_t rq, int row0, int rows_per_plane, int ldq, int k0, bool in, int lane) {
    const int c = lane & 7;
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = (lane >> 3) + 8 * j;
        const int k = k0 + 8 * c;
        r[p][j] = ld_b128(rq, in && k < ldq ? ((p * rows_per_plane + row0 + row) * ldq + k) * 2 : OOB, 0);
      }
  }
  __device__ __forceinline__ void store(char *tile, int lane) const {      // tile: NP planes of 4 KB
    const int c = lane & 7;
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int j = 0; j < 4; ++j) *(u32x4 *)(tile + p * 4096 + tile_off((lane >> 3) + 8 * j, c)) = r[p][j];
  }
};

template <int NP>
__global__ __launch_bounds__(256) void rlif_step_forward_kernel(const uint8_t *__restrict__ S, const float *__restrict__ I,
                                                                const float *__restrict__ V, float *__restrict__ Vn,
                                                                uint8_t *__restrict__ Sn,
                                                                const uint16_t *__restrict__ QRf, int ldqr,
                                                                long long qr_plane, int B, int N, int ld,
                                                                const float *__restrict__ beta_v, float theta) {
  constexpr int PF = NP == 1 ? 4 : 2;                    // tiles in flight per wavefront
  __shared__ float red[4][16][64];
  __shared__ __align__(16) char tiles[4][(NP + 1) * 4096];
  const RlifStepMap m = rlif_step_map((N + 31) / 32, (B + 31) / 32);
  if (!m.live) return;                                   // whole workgroup
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = m.st * 32 + (lane & 31);
  const unsigned bytes = (unsigned)B * ld * 4u;
  const rsrc_t rS = make_rsrc(S, bytes / 4), rQ = make_rsrc(QRf, (unsigned)(NP * qr_plane * 2));
  const int ktiles = (ld + 63) / 64, per = (ktiles + 3) / 4;
  const int kt0 = w * per, kt1 = min(ktiles, kt0 + per);
  const int rows_per_plane = (int)(qr_plane / ldqr);
  char *const wt = tiles[w], *const st = tiles[w] + NP * 4096;

  // operands of the update do not depend on the product: fetch them first
  const int n = m.nt * 32 + 8 * w + 4 * (lane >> 5);
  const bool upd = b < B && n < ld;
  const size_t o = upd ? (size_t)b * ld + n : 0;
  const float4 cur = *(const float4 *)(I + o), v = *(const float4 *)(V + o);
  const uint32_t sp = *(const uint32_t *)(S + o);
  const float4 be = *(const float4 *)(beta_v + (upd ? n : 0));

  // spike tile: 32 samples x 64 bytes, two 16-byte loads (lane: sample lane/4 + 16j, chunk lane%4)
  RlifWeightTile<NP> wr[PF];
  u32x4 sr[PF][2];
  auto fetch = [&](int d, int kt) {
    const bool in = kt < kt1;
    wr[d].load(rQ, m.nt * 32, rows_per_plane, ldqr, kt * 64, in, lane);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int sb = m.st * 32 + (lane >> 2) + 16 * j, k = kt * 64 + 16 * (lane & 3);
      sr[d][j] = ld_b128(rS, in && sb < B && k < ld ? sb * ld + k : OOB, 0);
    }
  };
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  auto consume = [&](int d) {
    wave_sync();                                         // the tile's previous readers are done
    wr[d].store(wt, lane);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = (lane >> 2) + 16 * j;
      u32x4 lo, hi;                                      // 16 spike bytes -> 16 bfloat16
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t x = sr[d][j][i];
        const uint32_t p0 = spikes2_to_bf16(__builtin_amdgcn_perm(0u, x, 0x0C010C00u));
        const uint32_t p1 = spikes2_to_bf16(__builtin_amdgcn_perm(0u, x, 0x0C030C02u));
        if (i < 2) { lo[2 * i] = p0; lo[2 * i + 1] = p1; } else { hi[2 * (i - 2)] = p0; hi[2 * (i - 2) + 1] = p1; }
      }
      *(u32x4 *)(st + tile_off(row, 2 * (lane & 3))) = lo;
      *(u32x4 *)(st + tile_off(row, 2 * (lane & 3) + 1)) = hi;
    }
    wave_sync();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int chunk = 2 * ks + (lane >> 5);
      const bf16x8 sf = *(const bf16x8 *)(st + tile_off(lane & 31, chunk));
#pragma unroll
      for (int p = NP - 1; p >= 0; --p) {
        const bf16x8 wf = *(const bf16x8 *)(wt + p * 4096 + tile_off(lane & 31, chunk));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, sf, acc, 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int d = 0; d < PF; ++d) fetch(d, kt0 + d);
  for (int kt = kt0; kt < kt1; kt += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      if (kt + d < kt1) consume(d);
      fetch(d, kt + d + PF);
    }
  }
  const f32x4 sum = rlif_reduce(acc, red, w, lane);
  if (upd) {
    const float c4[4] = {cur.x, cur.y, cur.z, cur.w}, v4[4] = {v.x, v.y, v.z, v.w}, b4[4] = {be.x, be.y, be.z, be.w};
    float vn[4];
    uint32_t out = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float s = (float)((sp >> (8 * i)) & 1u);
      vn[i] = b4[i] * v4[i] + c4[i] + sum[i] - theta * s;
      out |= (vn[i] > theta ? 1u : 0u) << (8 * i);
    }
    *(float4 *)(Vn + o) = make_float4(vn[0], vn[1], vn[2], vn[3]);
    *(uint32_t *)(Sn + o) = out;
  }
}

// One reverse step: gn = beta g + surr(V_t - theta) (dS_t - theta g + g R^T); the words of g
// (dI_t: hi/lo pairs with bfloat16 weights, fp32 bits otherwise) are the column operand.
template <int NP, int SURR>
__global__ __launch_bounds__(256) void rlif_step_reverse_kernel(const uint32_t *__restrict__ Gw, const float *__restrict__ G,
                                                                const float *__restrict__ dS, const float *__restrict__ V,
                                                                float *__restrict__ Gn, uint32_t *__restrict__ dIn,
                                                                const uint16_t *__restrict__ QRb, int ldqr,
                                                                long long qr_plane, int B, int N, int ld,
                                                                const float *__restrict__ beta_v, float theta, float slope,
                                                                float *__restrict__ db_part) {
  constexpr int GP = NP == 1 ? 2 : 3;
  constexpr bool HL = NP == 1;
  constexpr int PF = 2;
  __shared__ float red[4][16][64];
  __shared__ __align__(16) char tiles[4][(NP + GP) * 4096];
  const RlifStepMap m = rlif_step_map((N + 31) / 32, (B + 31) / 32);
  if (!m.live) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = m.st * 32 + (lane & 31);
  const unsigned bytes = (unsigned)B * ld * 4u;
  const rsrc_t rG = make_rsrc(Gw, bytes), rQ = make_rsrc(QRb, (unsigned)(NP * qr_plane * 2));
  const int ktiles = (ld + 63) / 64, per = (ktiles + 3) / 4;
  const int kt0 = w * per, kt1 = min(ktiles, kt0 + per);
  const int rows_per_plane = (int)(qr_plane / ldqr);
  char *const wt = tiles[w], *const gt = tiles[w] + NP * 4096;

  const int n = m.nt * 32 + 8 * w + 4 * (lane >> 5);
  const bool upd = b < B && n < ld;
  const size_t o = upd ? (size_t)b * ld + n : 0;
  const float4 ds = *(const float4 *)(dS + o), v = *(const float4 *)(V + o), g = *(const float4 *)(G + o);
  const float4 be = *(const float4 *)(beta_v + (upd ? n : 0));

  // tile of g words: 32 samples x 64 words, eight 16-byte loads (lane: sample lane/16 + 4j, words 4(lane%16)..)
  RlifWeightTile<NP> wr[PF];
  u32x4 gr[PF][8];
  auto fetch = [&](int d, int kt) {
    const bool in = kt < kt1;
    wr[d].load(rQ, m.nt * 32, rows_per_plane, ldqr, kt * 64, in, lane);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int sb = m.st * 32 + (lane >> 4) + 4 * j, k = kt * 64 + 4 * (lane & 15);
      gr[d][j] = ld_b128(rG, in && sb < B && k < ld ? (sb * ld + k) * 4 : OOB, 0);
    }
  };
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  auto consume = [&](int d) {
    wave_sync();
    wr[d].store(wt, lane);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = (lane >> 4) + 4 * j;
      const int off = tile_off(row, (lane & 15) >> 1) + 8 * (lane & 1);   // four bfloat16 = 8 bytes
      const u32x4 x = gr[d][j];
#pragma unroll
      for (int q = 0; q < GP; ++q) {
        u32x2 pl;
        if (HL) {
          pl[0] = q == 0 ? (x[0] & 0xFFFFu) | (x[1] << 16) : (x[0] >> 16) | (x[1] & 0xFFFF0000u);
          pl[1] = q == 0 ? (x[2] & 0xFFFFu) | (x[3] << 16) : (x[2] >> 16) | (x[3] & 0xFFFF0000u);
        } else {
          pl[0] = pack2(bf16_piece(__uint_as_float(x[0]), q), bf16_piece(__uint_as_float(x[1]), q));
          pl[1] = pack2(bf16_piece(__uint_as_float(x[2]), q), bf16_piece(__uint_as_float(x[3]), q));
        }
        *(u32x2 *)(gt + q * 4096 + off) = pl;
      }
    }
    wave_sync();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int chunk = 2 * ks + (lane >> 5);
      bf16x8 wf[NP], gf[GP];
#pragma unroll
      for (int p = 0; p < NP; ++p) wf[p] = *(const bf16x8 *)(wt + p * 4096 + tile_off(lane & 31, chunk));
#pragma unroll
      for (int q = 0; q < GP; ++q) gf[q] = *(const bf16x8 *)(gt + q * 4096 + tile_off(lane & 31, chunk));
      // smallest products first
#pragma unroll
      for (int sum = NP + GP - 2; sum >= 0; --sum)
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int q = sum - p;
          if (q >= 0 && q < GP && (NP == 1 || p + q < 3))
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[p], gf[q], acc, 0, 0, 0);
        }
    }
  };
#pragma unroll
  for (int d = 0; d < PF; ++d) fetch(d, kt0 + d);
  for (int kt = kt0; kt < kt1; kt += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      if (kt + d < kt1) consume(d);
      fetch(d, kt + d + PF);
    }
  }
  const f32x4 sum = rlif_reduce(acc, red, w, lane);
  if (upd) {
    const float d4[4] = {ds.x, ds.y, ds.z, ds.w}, v4[4] = {v.x, v.y, v.z, v.w}, g4[4] = {g.x, g.y, g.z, g.w};
    const float b4[4] = {be.x, be.y, be.z, be.w};
    float gn[4];
    uint32_t wd[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float q = d4[i] - theta * g4[i] + sum[i];
      gn[i] = b4[i] * g4[i] + surr_rcp<SURR>(slope, v4[i] - theta) * q;
      wd[i] = HL ? pack_hl(gn[i]) : __float_as_uint(gn[i]);
    }
    if (db_part) {                                     // dL/dbeta per sample, accumulated over the steps
      float4 acc4 = *(float4 *)(db_part + o);
      acc4.x += g4[0] * v4[0]; acc4.y += g4[1] * v4[1]; acc4.z += g4[2] * v4[2]; acc4.w += g4[3] * v4[3];
      *(float4 *)(db_part + o) = acc4;
    }
    *(float4 *)(Gn + o) = make_float4(gn[0], gn[1], gn[2], gn[3]);
    if (dIn) *(uint4 *)(dIn + o) = make_uint4(wd[0], wd[1], wd[2], wd[3]);
  }
}

// I, V [T][B][ld] fp32, S [T][B][ld] bytes; QRf[plane][to][from] bfloat16.
static hipError_t rlif_forward(hipStream_t st, bool fp32, int T, int B, int N, int ld, const float *I, float *V,
                               uint8_t *S, const uint16_t *QRf, int ldqr, long long qr_plane, const float *beta,
                               float theta) {
  if (ld <= 128) {                              // the whole time loop in one launch
    // Rows of a multiple of 16 neurons: tiles of 16 samples, eight wavefronts of 16 neurons, V_t
    // and S_t stored as whole rows.  Other widths: tiles of 32 samples, stores straight from the
    // accumulator layout.
    if (ld % 16 == 0) {
      const dim3 grid16((B + 15) / 16);
      if (fp32)
        hipLaunchKernelGGL((rlif_forward_fused16_kernel<3, 1>), grid16, dim3(512), 0, st, I, V, S, QRf, ldqr, qr_plane, T,
                           B, N, ld, beta, theta);
      else
        hipLaunchKernelGGL((rlif_forward_fused16_kernel<1, 1>), grid16, dim3(512), 0, st, I, V, S, QRf, ldqr, qr_plane, T,
                           B, N, ld, beta, theta);
      return hipGetLastError();
    }
    const dim3 grid((B + 31) / 32), block(256);
    if (fp32)
      hipLaunchKernelGGL((rlif_forward_fused_kernel<3>), grid, block, 0, st, I, V, S, QRf, ldqr, qr_plane, T, B, N,
                         ld, beta, theta);
    else
      hipLaunchKernelGGL((rlif_forward_fused_kernel<1>), grid, block, 0, st, I, V, S, QRf, ldqr, qr_plane, T, B, N,
                         ld, beta, theta);
    return hipGetLastError();
  }
  const size_t stride = (size_t)B * ld;
  hipError_t e;
  if ((e = fill_zero(st, V, stride * 4)) != hipSuccess) return e;     // V_0 = 0
  if ((e = fill_zero(st, S, stride)) != hipSuccess) return e;         // hence S_0 = 0
  const dim3 grid(rlif_step_grid(N, B)), block(256);
  for (int t = 0; t + 1 < T; ++t) {
    const uint8_t *s = S + t * stride;
    const float *cur = I + t * stride, *v = V + t * stride;
    float *vn = V + (t + 1) * stride;
    uint8_t *sn = S + (t + 1) * stride;
    if (fp32)
      hipLaunchKernelGGL(rlif_step_forward_kernel<3>, grid, block, 0, st, s, cur, v, vn, sn, QRf, ldqr, qr_plane, B, N,
                         ld, beta, theta);
    else
      hipLaunchKernelGGL(rlif_step_forward_kernel<1>, grid, block, 0, st, s, cur, v, vn, sn, QRf, ldqr, qr_plane, B, N,
                         ld, beta, theta);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

// dS, V [T][B][ld] fp32; dI [T][B][ld] dwords (fp32, or HL with rounded weights); g0, g1
// [B][ld] fp32 scratch for dL/dV_{t+1}; QRb[plane][from][to] bfloat16.
static hipError_t rlif_reverse(hipStream_t st, bool fp32, int T, int B, int N, int ld, const float *dS, const float *V,
                               uint32_t *dI, float *g0, float *g1, const uint16_t *QRb, int ldqr,
                               long long qr_plane, const float *beta, float theta, int surrogate, float slope, float *db_part) {
  if (ld <= 128) {
    const dim3 grid((B + 15) / 16);
#define SNN_RLR(NP, SU)                                                                                         \
  hipLaunchKernelGGL((rlif_reverse_fused16_kernel<NP, SU, 1>), grid, dim3(512), 0, st, dS, V, dI, QRb, ldqr, qr_plane, \
                     T, B, N, ld, beta, theta, slope, db_part)
    if (fp32) {
      switch (surrogate) { case 0: SNN_RLR(3, 0); break; case 1: SNN_RLR(3, 1); break;
                           case 2: SNN_RLR(3, 2); break; case 3: SNN_RLR(3, 3); break;
                           case 4: SNN_RLR(3, 4); break; default: SNN_RLR(3, 5); break; }
    } else {
      switch (surrogate) { case 0: SNN_RLR(1, 0); break; case 1: SNN_RLR(1, 1); break;
                           case 2: SNN_RLR(1, 2); break; case 3: SNN_RLR(1, 3); break;
                           case 4: SNN_RLR(1, 4); break; default: SNN_RLR(1, 5); break; }
    }
#undef SNN_RLR
    return hipGetLastError();
  }
  const size_t stride = (size_t)B * ld;
  hipError_t e;
  if ((e = fill_zero(st, g0, stride * 4)) != hipSuccess) return e;                              // g_T = 0
  if (db_part && (e = fill_zero(st, db_part, stride * 4)) != hipSuccess) return e;              // accumulated step by step
  if ((e = fill_zero(st, dI + (size_t)(T - 1) * stride, stride * 4)) != hipSuccess) return e;   // dI_{T-1} = 0
  const dim3 grid(rlif_step_grid(N, B)), block(256);
  float *g[2] = {g0, g1};
  int cur = 0;
  for (int t = T - 1; t >= 0; --t) {
    const uint32_t *gw = dI + (size_t)t * stride;              // dI_t = g_{t+1}, in product form
    const float *ds = dS + t * stride, *v = V + t * stride;
    uint32_t *din = t > 0 ? dI + (size_t)(t - 1) * stride : nullptr;
#define SNN_RSR(NP, SU)                                                                                          \
  hipLaunchKernelGGL((rlif_step_reverse_kernel<NP, SU>), grid, block, 0, st, gw, g[cur], ds, v, g[cur ^ 1], din, QRb, \
                     ldqr, qr_plane, B, N, ld, beta, theta, slope, db_part)
    if (fp32) {
      switch (surrogate) { case 0: SNN_RSR(3, 0); break; case 1: SNN_RSR(3, 1); break;
                           case 2: SNN_RSR(3, 2); break; case 3: SNN_RSR(3, 3); break;
                           case 4: SNN_RSR(3, 4); break; default: SNN_RSR(3, 5); break; }
    } else {
      switch (surrogate) { case 0: SNN_RSR(1, 0); break; case 1: SNN_RSR(1, 1); break;
                           case 2: SNN_RSR(1, 2); break; case 3: SNN_RSR(1, 3); break;
                           case 4: SNN_RSR(1, 4); break; default: SNN_RSR(1, 5); break; }
    }
#undef SNN_RSR
    if ((e = hipGetLastError()) != hipSuccess) return e;
    cur ^= 1;
  }
  return hipSuccess;
}

}  // namespace snn
