// Time scans, readout, loss and parameter kernels of the training step, gfx950.
//
// The LIF scans are bound by HBM traffic: one thread owns VEC adjacent chains
// (b, n..n+VEC-1), keeps their state in registers for all T steps and streams the per-step
// rows.  Loads do not depend on the recurrence, so a block of U steps is fetched while the
// previous block is being integrated.
#pragma once
#include "common.hpp"

namespace snn {

// VEC adjacent fp32 / dword / byte values at lane offset `voff` (+ scalar offset `soff`).
template <int VEC, int POLICY = 0> __device__ __forceinline__ void ldv(float (&d)[VEC], rsrc_t r, int voff, int soff) {
  if (VEC == 1) d[0] = __uint_as_float(ld_b32<POLICY>(r, voff, soff));
  else if (VEC == 2) { const u32x2 v = ld_b64<POLICY>(r, voff, soff); d[0] = __uint_as_float(v[0]); d[1] = __uint_as_float(v[1]); }
  else { const u32x4 v = ld_b128<POLICY>(r, voff, soff);
#pragma unroll
    for (int i = 0; i < VEC; ++i) d[i] = __uint_as_float(v[i]); }
}
template <int VEC> __device__ __forceinline__ void stv(rsrc_t r, int voff, int soff, const uint32_t (&d)[VEC]) {
  if (VEC == 1) st_b32(r, voff, soff, d[0]);
  else if (VEC == 2) { u32x2 v; v[0] = d[0]; v[1] = d[1]; st_b64(r, voff, soff, v); }
  else { u32x4 v;
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = d[i];
    st_b128(r, voff, soff, v); }
}
template <int VEC> __device__ __forceinline__ void st_spikes(rsrc_t r, int voff, int soff, const uint32_t (&s)[VEC]) {
  if (VEC == 1) st_b8(r, voff, soff, s[0]);
  else if (VEC == 2) st_b16(r, voff, soff, s[0] | (s[1] << 8));
  else st_b32(r, voff, soff, s[0] | (s[1] << 8) | (s[2] << 16) | (s[3] << 24));
}

// ---------------------------------------------------------------- LIF forward (Eq. 1-2)
// S_t = [V_t > theta]; store V_t, S_t; V_{t+1} = beta V_t + I_t - theta S_t; V_0 = 0.
// `stride` = B * ld elements between time steps; threads cover the stride (padding
// columns included: their currents are zero, so they stay silent).  A lane's offset into a
// time row never changes, the row offset is scalar: no per-access vector address
// arithmetic.  Whole blocks of 2U steps run without a branch; fetches past the end re-read
// the last row (never used), the ragged tail runs guarded.
// POL: cache policy of the loads.  Tensors far larger than the caches (L2 8 x 4 MiB, 256 MiB
// memory-side) are read non-temporally: 8 % (forward) and 11 % (reverse) faster at 537 MB per
// tensor.  Smaller ones are still warm from the kernel that wrote them, and the same hint
// costs 10 % there.
// ADAPT: neurons with an adaptive firing threshold.  A second state A (A_0 = 0) raises the
// threshold, theta_t = theta + A_t; the spike and the reset take theta_t, then
// A_{t+1} = gamma A_t + kappa S_t.  A_t is stored beside V_t (the reverse scan needs both).
template <int VEC, int U, int POL, bool ADAPT>
__global__ __launch_bounds__(256) void lif_forward_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                          uint8_t *__restrict__ S, int T, int stride,
                                                          const float *__restrict__ beta_v, int ld, float theta,
                                                          float *__restrict__ A, float gamma, float kappa) {
  const int p = (blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (p >= stride) return;
  float beta[VEC];                                   // one decay per neuron (column p % ld)
#pragma unroll
  for (int i = 0; i < VEC; ++i) beta[i] = beta_v[p % ld + i];
  const rsrc_t rI = make_rsrc(I, (unsigned)T * stride * 4u), rV = make_rsrc(V, (unsigned)T * stride * 4u);
  const rsrc_t rS = make_rsrc(S, (unsigned)T * stride);
  const rsrc_t rA = make_rsrc(A, ADAPT ? (unsigned)T * stride * 4u : 0u);
  const int vo4 = p * 4, vo1 = p, row4 = stride * 4;
  float v[VEC], ad[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) v[i] = ad[i] = 0.f;
  float a[U][VEC], b[U][VEC];

  auto fetch = [&](float (&buf)[U][VEC], int t0) {
#pragma unroll
    for (int u = 0; u < U; ++u) ldv<VEC, POL>(buf[u], rI, vo4, min(t0 + u, T - 1) * row4);
  };
  auto step = [&](const float (&cur)[VEC], int t) {
    uint32_t s[VEC], w[VEC];
    float thr[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      thr[i] = ADAPT ? theta + ad[i] : theta;
      s[i] = v[i] > thr[i] ? 1u : 0u;
      w[i] = __float_as_uint(v[i]);
    }
    stv<VEC>(rV, vo4, t * row4, w);
    st_spikes<VEC>(rS, vo1, t * stride, s);
    if (ADAPT) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) w[i] = __float_as_uint(ad[i]);
      stv<VEC>(rA, vo4, t * row4, w);
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      v[i] = beta[i] * v[i] + cur[i] - (s[i] ? thr[i] : 0.f);
      if (ADAPT) ad[i] = gamma * ad[i] + (s[i] ? kappa : 0.f);
    }
  };
  fetch(a, 0);
  int t0 = 0;
  for (; t0 + 2 * U <= T; t0 += 2 * U) {
    fetch(b, t0 + U);
#pragma unroll
    for (int u = 0; u < U; ++u) step(a[u], t0 + u);
    fetch(a, t0 + 2 * U);
#pragma unroll
    for (int u = 0; u < U; ++u) step(b[u], t0 + U + u);
  }
  if (t0 < T) {                                     // fewer than 2U steps left; a holds t0..
    fetch(b, t0 + U);
#pragma unroll
    for (int u = 0; u < U; ++u) if (t0 + u < T) step(a[u], t0 + u);
#pragma unroll
    for (int u = 0; u < U; ++u) if (t0 + U + u < T) step(b[u], t0 + U + u);
  }
}

// ---------------------------------------------------------------- LIF reverse, fused surrogate
// g = 0; for t = T-1..0: dI_t = g; g = beta g + surr(V_t - theta) (dS_t - theta g).
// With db_part: also dL/dbeta per chain, sum_t g_{t+1} V_t (V_{t+1} = beta V_t + ..).
// dI is written as fp32 or, when HL, in the hi/lo form the bfloat16 products read.
// ADAPT (adaptive threshold, see lif_forward_kernel): with theta_t = theta + A_t and ga the
// gradient of A_{t+1}: q = dS_t - theta_t g + kappa ga; the spike decision's derivative is the
// surrogate at V_t - theta_t with respect to V_t and its negative with respect to A_t, so
// ga <- gamma ga - S_t g - surr q (S_t = [V_t > theta_t], the reset's factor) and
// g <- beta g + surr q.
template <int SURR> __device__ __forceinline__ float surr(float k, float x) {
  if (SURR == 0) { float d = 1.0f + k * fabsf(x); return 1.0f / (d * d); }
  if (SURR == 1) { float u = 1.5707963267948966f * k * x; return (0.5f * k) / (1.0f + u * u); }
  if (SURR == 2) { float s = 1.0f / (1.0f + __expf(-k * x)); return k * s * (1.0f - s); }
  if (SURR == 3) return fmaxf(0.0f, 1.0f - fabsf(k * x));
  if (SURR == 4) return fabsf(k * x) <= 1.0f ? 0.5f : 0.0f;      // boxcar
  return 1.0f;                                                   // straight-through
}

// The surrogates with the hardware reciprocal (1 ulp) instead of an IEEE division: for the
// kernels where the surrogate's arithmetic, not memory, is what a step waits for (the one-launch
// layer reverse: the division alone took 1.6 us per block of 64 steps; the recurrent reverse
// kernel: sixteen divisions per lane and step).
template <int SURR> __device__ __forceinline__ float surr_rcp(float k, float x) {
  if (SURR == 0) { const float d = 1.0f + k * fabsf(x); return __builtin_amdgcn_rcpf(d * d); }
  if (SURR == 1) { const float u = 1.5707963267948966f * k * x; return (0.5f * k) * __builtin_amdgcn_rcpf(1.0f + u * u); }
  if (SURR == 2) { const float s = __builtin_amdgcn_rcpf(1.0f + __expf(-k * x)); return k * s * (1.0f - s); }
  return surr<SURR>(k, x);
}

template <int VEC, int U, int SURR, bool HL, int POL, bool ADAPT>
__global__ __launch_bounds__(256) void lif_reverse_kernel(const float *__restrict__ dS, const float *__restrict__ V,
                                                          uint32_t *__restrict__ dI, int T, int stride,
                                                          const float *__restrict__ beta_v, int ld, float theta,
                                                          float slope, float *__restrict__ db_part,
                                                          const float *__restrict__ A, float gamma, float kappa) {
  const int p = (blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (p >= stride) return;
  float beta[VEC], db[VEC];                          // decay per neuron; sum over t of g_{t+1} V_t
#pragma unroll
  for (int i = 0; i < VEC; ++i) { beta[i] = beta_v[p % ld + i]; db[i] = 0.f; }
  const unsigned bytes = (unsigned)T * stride * 4u;
  const rsrc_t rdS = make_rsrc(dS, bytes), rV = make_rsrc(V, bytes), rdI = make_rsrc(dI, bytes);
  const rsrc_t rA = make_rsrc(A, ADAPT ? bytes : 0u);
  const int vo4 = p * 4, row4 = stride * 4;
  constexpr int UA = ADAPT ? U : 1;                  // the adaptation's rows are only fetched when it exists
  float g[VEC], ga[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) g[i] = ga[i] = 0.f;
  float a_ds[U][VEC], a_v[U][VEC], b_ds[U][VEC], b_v[U][VEC], a_a[UA][VEC], b_a[UA][VEC];

  // a block covers steps thi, thi-1, .., thi-U+1 (clamped at 0: re-reads, never used)
  auto fetch = [&](float (&bds)[U][VEC], float (&bv)[U][VEC], float (&ba)[UA][VEC], int thi) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int so = max(thi - u, 0) * row4;
      ldv<VEC, POL>(bds[u], rdS, vo4, so);
      ldv<VEC, POL>(bv[u], rV, vo4, so);
      if (ADAPT) ldv<VEC, POL>(ba[u % UA], rA, vo4, so);
    }
  };
  auto step = [&](const float (&ds)[VEC], const float (&vv)[VEC], const float (&aa)[VEC], int t) {
    uint32_t w[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) w[i] = HL ? pack_hl(g[i]) : __float_as_uint(g[i]);
    stv<VEC>(rdI, vo4, t * row4, w);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      db[i] += g[i] * vv[i];
      if (ADAPT) {
        const float thr = theta + aa[i], x = vv[i] - thr;
        const float sq = surr_rcp<SURR>(slope, x) * (ds[i] - thr * g[i] + kappa * ga[i]);
        ga[i] = gamma * ga[i] - (x > 0.f ? g[i] : 0.f) - sq;
        g[i] = beta[i] * g[i] + sq;
      } else {
        g[i] = beta[i] * g[i] + surr_rcp<SURR>(slope, vv[i] - theta) * (ds[i] - theta * g[i]);
      }
    }
  };
  fetch(a_ds, a_v, a_a, T - 1);
  int thi = T - 1;
  for (; thi - 2 * U + 1 >= 0; thi -= 2 * U) {
    fetch(b_ds, b_v, b_a, thi - U);
#pragma unroll
    for (int u = 0; u < U; ++u) step(a_ds[u], a_v[u], a_a[u % UA], thi - u);
    fetch(a_ds, a_v, a_a, thi - 2 * U);
#pragma unroll
    for (int u = 0; u < U; ++u) step(b_ds[u], b_v[u], b_a[u % UA], thi - U - u);
  }
  if (thi >= 0) {
    fetch(b_ds, b_v, b_a, thi - U);
#pragma unroll
    for (int u = 0; u < U; ++u) if (thi - u >= 0) step(a_ds[u], a_v[u], a_a[u % UA], thi - u);
#pragma unroll
    for (int u = 0; u < U; ++u) if (thi - U - u >= 0) step(b_ds[u], b_v[u], b_a[u % UA], thi - U - u);
  }
  if (db_part) {                                     // per sample; summed over the batch by the reduction launch
#pragma unroll
    for (int i = 0; i < VEC; ++i) db_part[p + i] = db[i];
  }
}

// ---------------------------------------------------------------- LI readout, max over time
// y_t = beta y_{t-1} + J_t, y_{-1} = 0; z = max_t y_t; t* = first maximiser.
// `integral`: z = sum_t y_t instead (t* = 0, not used).
__global__ __launch_bounds__(256) void readout_forward_kernel(const float *__restrict__ J, float *__restrict__ Y,
                                                              float *__restrict__ z, int *__restrict__ tstar,
                                                              int T, int stride, const float *__restrict__ beta_v,
                                                              int ld, int integral) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= stride) return;
  const float beta = beta_v[p % ld];
  float y = 0.f, best = -INFINITY, sum = 0.f;
  int tb = 0;
#pragma unroll 8
  for (int t = 0; t < T; ++t) {
    y = beta * y + J[(size_t)t * stride + p];
    Y[(size_t)t * stride + p] = y;
    sum += y;
    if (y > best) { best = y; tb = t; }
  }
  z[p] = integral ? sum : best;
  tstar[p] = integral ? 0 : tb;
}

// Softmax cross-entropy, one wavefront per sample: lanes stride over the classes and the
// maximum and the sum are reduced across the wavefront.
__global__ __launch_bounds__(256) void cross_entropy_kernel(const float *__restrict__ z, const int *__restrict__ labels,
                                                            float *__restrict__ loss_b, float *__restrict__ dz,
                                                            int B, int C, int ldc, int *__restrict__ err) {
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (b >= B) return;
  const float *zb = z + (size_t)b * ldc;
  float m = -INFINITY;
  for (int c = lane; c < C; c += 64) m = fmaxf(m, zb[c]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  float sum = 0.f;
  for (int c = lane; c < C; c += 64) sum += expf(zb[c] - m);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  int lab = labels[b];
  if (lab < 0 || lab >= C) { if (lane == 0) atomicOr(err, 1); lab = 0; }
  if (lane == 0) loss_b[b] = m + logf(sum) - zb[lab];
  const float inv = 1.0f / sum, invB = 1.0f / (float)B;
  for (int c = lane; c < C; c += 64)
    dz[(size_t)b * ldc + c] = (expf(zb[c] - m) * inv - (c == lab ? 1.f : 0.f)) * invB;
}

// Orders the LDS traffic of one wavefront: lanes exchange data through LDS without a
// workgroup barrier (LDS operations of a wavefront execute in order); the fences keep the
// compiler from moving accesses across the exchange point.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------- LIF forward below the readout
// The forward scan of the last spiking layer, which also forms the readout's currents
// J_t = S_t W of the steps it has just produced: that product has only C <= 32 columns, a
// launch of its own reads all spikes again for 3 MB of result.  A workgroup owns one sample:
// NW wavefronts of 64 chains each (ld = 64 NW).  Per block of 16 steps a wavefront writes its
// spikes as bfloat16 into a private 16 x 64 LDS tile, reads them back as the A operand of
// 16x16x32 MFMAs (rows = steps, k = its 64 neurons; B = the rounded readout weights of those
// neurons, lane: class lane%16 of a group of 16, neurons 8 (lane/16) .. +7 of a half), and
// the per-wavefront partial sums are added across the workgroup in a fixed order.
// Wq: bfloat16 [class][neuron] rows of ldq elements, zero beyond the C classes and N neurons.
template <int NW, int POL>
__global__ __launch_bounds__(64 * NW) void lif_forward_top_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                                  uint8_t *__restrict__ S, float *__restrict__ J,
                                                                  int ldc, const uint16_t *__restrict__ Wq, int ldq,
                                                                  int q_rows, int T, int B, int stride,
                                                                  const float *__restrict__ beta_v, float theta) {
  constexpr int U = 16, LD = 64 * NW, TP = 144;             // steps per block; row length; tile pitch in bytes
  __shared__ __attribute__((aligned(16))) char tile[NW][U * TP];
  __shared__ float red[2][NW][U][32];                       // double-buffered: one barrier per block
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = blockIdx.x, n = 64 * w + lane;
  const int p = b * LD + n;
  const float beta = beta_v[n];
  const unsigned bytes = (unsigned)T * stride * 4u;
  const rsrc_t rI = make_rsrc(I, bytes), rV = make_rsrc(V, bytes), rS = make_rsrc(S, (unsigned)T * stride);
  const rsrc_t rW = make_rsrc(Wq, (unsigned)q_rows * ldq * 2u);
  const int vo4 = p * 4, row4 = stride * 4;
  const int kg = lane >> 4;

  bf16x8 wf[2][2];                                          // [class group][neuron half]
#pragma unroll
  for (int cg = 0; cg < 2; ++cg)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int cls = 16 * cg + (lane & 15);
      wf[cg][ks] = __builtin_bit_cast(bf16x8, ld_b128(rW, cls < q_rows ? (cls * ldq + 64 * w + 32 * ks + 8 * kg) * 2 : OOB, 0));
    }

  float v = 0.f;
  float a[U], bb[U];
  auto fetch = [&](float (&buf)[U], int t0) {
#pragma unroll
    for (int u = 0; u < U; ++u) buf[u] = __uint_as_float(ld_b32<POL>(rI, vo4, min(t0 + u, T - 1) * row4));
  };
  // 16 steps from t0; steps beyond T leave no trace in memory and put zeros into the tile
  auto block = [&](const float (&cur)[U], int t0, int par) {
    char *const mine = tile[w];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u;
      const bool live = t < T;
      const uint32_t s = live && v > theta ? 1u : 0u;
      if (live) {
        st_b32(rV, vo4, t * row4, __float_as_uint(v));
        st_b8(rS, p, t * stride, s);
        v = beta * v + cur[u] - (s ? theta : 0.f);
      }
      *(uint16_t *)(mine + u * TP + 2 * lane) = s ? 0x3F80 : 0;
    }
    wave_sync();
    bf16x8 af[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) af[ks] = *(const bf16x8 *)(mine + (lane & 15) * TP + (32 * ks + 8 * kg) * 2);
#pragma unroll
    for (int cg = 0; cg < 2; ++cg) {
      f32x4 d = {0.f, 0.f, 0.f, 0.f};
      d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[0], wf[cg][0], d, 0, 0, 0);
      d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[1], wf[cg][1], d, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) red[par][w][4 * kg + r][16 * cg + (lane & 15)] = d[r];
    }
    __syncthreads();
    // J[t0 + step][b][c]: thread -> class tid % 32, steps tid / 32 + (2 NW) k
    {
      const int c = threadIdx.x & 31;
#pragma unroll
      for (int st = threadIdx.x >> 5; st < U; st += 2 * NW) {
        float sum = red[par][0][st][c];
#pragma unroll
        for (int x = 1; x < NW; ++x) sum += red[par][x][st][c];
        if (c < ldc && t0 + st < T) J[((size_t)(t0 + st) * B + b) * ldc + c] = sum;
      }
    }
  };
  fetch(a, 0);
  int t0 = 0;
  for (; t0 + 2 * U <= T; t0 += 2 * U) {
    fetch(bb, t0 + U);
    block(a, t0, 0);
    fetch(a, t0 + 2 * U);
    block(bb, t0 + U, 1);
  }
  if (t0 < T) {
    fetch(bb, t0 + U);
    block(a, t0, 0);
    if (t0 + U < T) block(bb, t0 + U, 1);
  }
}

// ---------------------------------------------------------------- LIF reverse below a narrow layer
// The reverse scan of a spiking layer that takes dS_t = dX_t W^T from the current gradients dX
// of the layer above itself instead of reading it from memory, for a layer above of at most
// 128 columns (32 KS): the readout (dX = dJ, C <= 32 classes) or a narrow spiking layer.  With
// so few terms per element a separate product launch writes 4 bytes per element and this scan
// reads them back for nothing (a third of its traffic).  One wavefront owns 64 chains, all of
// one sample (ld is a multiple of 64 here), and per block of 16 steps forms the 16 x 64 block
// of dS with 16x16x32 bfloat16 MFMAs:
//   A  rows = the 16 steps, k = column of the layer above: the hi and the lo halves of the dX
//      words of this sample (lane: step lane%16, columns 32 ks + 8 (lane/16) .. +7), two
//      passes, lo first
//   B  columns = 16 chains, k as in A: the rounded weights W[n][k] (lane: chain lane%16 of the
//      group), fetched once per group of 16 chains
//   D  lane holds chain lane%16 of the group at steps 4 (lane/16) .. +3
// The block goes through 4 KiB of LDS private to the wavefront and comes back with one chain
// per lane; after that the kernel is lif_reverse_kernel with one chain per lane.
// dX: hi/lo words [T][B][ldc], Wq: bfloat16 [ld rows][ldq] (row n = neuron of this layer),
// zero beyond the valid columns.
template <int KS, int SURR, int POL>
__global__ __launch_bounds__(256) void lif_reverse_top_kernel(const uint32_t *__restrict__ dX, int ldc,
                                                             const uint16_t *__restrict__ Wq, int ldq,
                                                             const float *__restrict__ V, uint32_t *__restrict__ dI,
                                                             int T, int B, int stride,
                                                             const float *__restrict__ beta_v, int ld, float theta,
                                                             float slope, float *__restrict__ db_part) {
  constexpr int U = 16;                                     // steps per block (32 measured slower)
  __shared__ float blks[4][U][64];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float (&blk)[U][64] = blks[wv];
  // The wavefronts of a workgroup (1, 2 or 4) are neighbours in the row and so belong to one
  // sample: they fetch the same dX words, the second fetch is served by the CU's cache.  (As
  // workgroups of their own they land on different XCDs and each fetch goes to memory.)
  const int p0 = (blockIdx.x * (blockDim.x >> 6) + wv) * 64, p = p0 + lane;   // stride is a multiple of 64
  const int b = p0 / ld, n0 = p0 % ld;                     // one sample per wavefront
  const float beta = beta_v[n0 + lane];
  float db = 0.f, g = 0.f;
  const unsigned bytes = (unsigned)T * stride * 4u;
  const rsrc_t rV = make_rsrc(V, bytes), rdI = make_rsrc(dI, bytes);
  const rsrc_t rX = make_rsrc(dX, (unsigned)T * B * ldc * 4u), rW = make_rsrc(Wq, (unsigned)ld * ldq * 2u);
  const int vo4 = p * 4, row4 = stride * 4;
  const int kg = lane >> 4;

  bf16x8 wf[4][KS];                                         // B fragments: the weights of 4 x 16 chains
#pragma unroll
  for (int grp = 0; grp < 4; ++grp)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = 32 * ks + 8 * kg;
      wf[grp][ks] = __builtin_bit_cast(bf16x8, ld_b128(rW, k < ldq ? ((n0 + 16 * grp + (lane & 15)) * ldq + k) * 2 : OOB, 0));
    }

  // dX words of a block: steps thi-15 .. thi of sample b (row lane%16), columns 32 ks + 8 kg .. +7
  const int xrow = B * ldc * 4;
  auto fetch_x = [&](u32x4 (&x)[KS][2], int thi) {
    const int t = thi - (U - 1) + (lane & 15);             // the row differs per lane: all of it in the lane offset
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = 32 * ks + 8 * kg;
      const int xo = t >= 0 && k + 7 < ldc ? t * xrow + (b * ldc + k) * 4 : OOB;
      x[ks][0] = ld_b128(rX, xo, 0);
      x[ks][1] = ld_b128(rX, xo == OOB ? OOB : xo + 16, 0);
    }
  };
  auto fetch_v = [&](float (&v)[U], int thi) {
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __uint_as_float(ld_b32<POL>(rV, vo4, max(thi - u, 0) * row4));
  };
  // dS of the block with last step thi: ds[u] = dS at step thi - u of this lane's chain
  auto spikes_grad = [&](const u32x4 (&x)[KS][2], float (&ds)[U]) {
    bf16x8 hi[KS], lo[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 (&j)[2] = x[ks];
      u32x4 h, l;
      h.x = __builtin_amdgcn_perm(j[0].y, j[0].x, 0x05040100u); l.x = __builtin_amdgcn_perm(j[0].y, j[0].x, 0x07060302u);
      h.y = __builtin_amdgcn_perm(j[0].w, j[0].z, 0x05040100u); l.y = __builtin_amdgcn_perm(j[0].w, j[0].z, 0x07060302u);
      h.z = __builtin_amdgcn_perm(j[1].y, j[1].x, 0x05040100u); l.z = __builtin_amdgcn_perm(j[1].y, j[1].x, 0x07060302u);
      h.w = __builtin_amdgcn_perm(j[1].w, j[1].z, 0x05040100u); l.w = __builtin_amdgcn_perm(j[1].w, j[1].z, 0x07060302u);
      hi[ks] = __builtin_bit_cast(bf16x8, h);
      lo[ks] = __builtin_bit_cast(bf16x8, l);
    }
    wave_sync();                                            // the previous block has been read
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo[ks], wf[grp][ks], d, 0, 0, 0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi[ks], wf[grp][ks], d, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) blk[4 * kg + r][16 * grp + (lane & 15)] = d[r];
    }
    wave_sync();
#pragma unroll
    for (int u = 0; u < U; ++u) ds[u] = blk[U - 1 - u][lane];
  };
  auto step = [&](float ds, float vv, int t) {
    st_b32(rdI, vo4, t * row4, pack_hl(g));
    db += g * vv;
    g = beta * g + surr_rcp<SURR>(slope, vv - theta) * (ds - theta * g);
  };

  // The dS block of the next 16 steps is formed before the current 16 are scanned, so that its
  // trip through the MFMA units and LDS runs under the scan's arithmetic; the dX words are
  // fetched two blocks ahead, the potentials one.  (Blocks beyond step 0 read nothing.)
  u32x4 xa[KS][2], xb[KS][2];
  float va[U], vb[U], dsa[U], dsb[U];
  fetch_x(xa, T - 1);
  fetch_v(va, T - 1);
  fetch_x(xb, T - 1 - U);
  spikes_grad(xa, dsa);
  int thi = T - 1;
  for (; thi - 2 * U + 1 >= 0; thi -= 2 * U) {
    fetch_v(vb, thi - U);
    fetch_x(xa, thi - 2 * U);
    spikes_grad(xb, dsb);
#pragma unroll
    for (int u = 0; u < U; ++u) step(dsa[u], va[u], thi - u);
    fetch_v(va, thi - 2 * U);
    fetch_x(xb, thi - 3 * U);
    spikes_grad(xa, dsa);
#pragma unroll
    for (int u = 0; u < U; ++u) step(dsb[u], vb[u], thi - U - u);
  }
  if (thi >= 0) {
    fetch_v(vb, thi - U);
    spikes_grad(xb, dsb);
#pragma unroll
    for (int u = 0; u < U; ++u) if (thi - u >= 0) step(dsa[u], va[u], thi - u);
#pragma unroll
    for (int u = 0; u < U; ++u) if (thi - U - u >= 0) step(dsb[u], vb[u], thi - U - u);
  }
  if (db_part) db_part[p] = db;
}

// Readout scan, loss and readout reverse in one launch, for C <= 64.
//
// Chains: a workgroup holds SPB = 64/CW samples, CW lanes each (CW = power of two >= ld), one
// lane per (b, c) chain; the softmax is reduced across the CW lanes of a sample.
//
// Time: the LI readout has no threshold and no reset, so y_t = beta y_{t-1} + J_t is linear
// in the state and can be cut in time.  The eight wavefronts of a workgroup all hold the same
// 64 chains; in every block of 128 steps wavefront w owns steps [16w, 16w+16).  It first
// integrates its steps from a zero state (e_w), the e_w are exchanged through LDS, the state
// entering its segment follows as c_w = beta^16 c_{w-1} + e_{w-1}, and the segment is then
// integrated for real from c_w, step by step as the sequential scan would.  A single
// wavefront issuing ~10 instructions per step is what bounds this kernel, hence the split.
// The first maximiser over time is found per wavefront and merged (larger value, then
// earlier step).  With the max over time, dJ_t = beta^(t*-t) dz for t <= t* and 0 after
// (the recursion h_t = beta h_{t+1} + dz [t == t*]); a wavefront enters its segment with the
// closed form and runs the recursion inside it.
//
// Memory: a wavefront can have 63 memory operations in flight, so global accesses are
// 16 bytes per lane and cover four time rows at once: lane i of the "memory" arrangement
// holds columns 4q..4q+3 of row r (r = i / LPR, q = i % LPR, LPR = SPB*ld/4 <= 16 lanes per
// row); a 1 KB LDS stage per access turns that into the chain arrangement and back.  Lanes
// without work address beyond the buffers: loads return zero, stores are dropped.
// Per-sample losses go to loss_b; their mean is taken by a later launch (the partial-sum
// reduction of the backward pass, or loss_mean_kernel when the loss is asked for first), in
// index order either way.
template <int CW, bool HL, bool INTEGRAL>
__global__ __launch_bounds__(512) void readout_loss_kernel(const float *__restrict__ J, float *__restrict__ Y,
                                                           float *__restrict__ z, int *__restrict__ tstar,
                                                           const int *__restrict__ labels, float *__restrict__ loss_b,
                                                           float *__restrict__ dz, int *__restrict__ err,
                                                           uint32_t *__restrict__ dJ, int T, int B, int C, int ldc,
                                                           const float *__restrict__ beta_v) {
  constexpr int SPB = 64 / CW;                        // samples per workgroup
  constexpr int NW = 8;                               // wavefronts = time segments per block
  constexpr int G = 4;                                // accesses (of four rows) per segment
  constexpr int SEG = 4 * G;                          // steps per segment
  constexpr int SB = NW * SEG;                        // steps per block
  __shared__ __align__(16) uint32_t stage[NW][G][256];   // one wavefront's rows in flight, in or out
  __shared__ float x_e[2][NW][64], x_best[NW][64];
  __shared__ int x_tb[NW][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int stride = B * ldc, row4 = stride * 4;
  const unsigned bytes = (unsigned)T * stride * 4u;
  const rsrc_t rJ = make_rsrc(J, bytes), rY = make_rsrc(Y, bytes), rdJ = make_rsrc(dJ, bytes);

  // chain arrangement
  const int c = lane % CW;
  const int s = lane / CW;
  const int b = blockIdx.x * SPB + s;
  const bool live = b < B && c < C;
  const bool staged = c < ldc;                        // has a slot in the stages
  const int slot = staged ? s * ldc + c : 0;
  const int p = live ? b * ldc + c : 0;
  // memory arrangement
  const int lpr = SPB * ldc / 4;
  const int mr = lane / lpr, mq = lane - mr * lpr;
  const int mchain = blockIdx.x * SPB * ldc + 4 * mq;
  const bool mvalid = mr < 4 && mchain < stride;
  const int mvo = mvalid ? mr * row4 + mchain * 4 : OOB;
  const int mslot = mvalid ? mr * 64 + 4 * mq : 0;    // dword index in a stage
  auto mem_off = [&](int t0) { return t0 + mr < T ? mvo : OOB; };   // rows past the end: no access

  const int lab_in = b < B ? labels[b] : 0;
  const float beta = c < ldc ? beta_v[c] : 0.f;       // the class's decay
  float bseg = beta;                                  // beta^SEG
#pragma unroll
  for (int i = 0; i < 4; ++i) bseg *= bseg;
  static_assert(SEG == 16, "bseg is beta^16");

  float y_in = 0.f, best = -INFINITY, ysum = 0.f;     // y_in: state entering the block
  int tb = 0;
  for (int sb0 = 0, par = 0; sb0 < T; sb0 += SB, par ^= 1) {
    const int t0 = sb0 + SEG * w;
    u32x4 raw[G];
#pragma unroll
    for (int g = 0; g < G; ++g) raw[g] = ld_b128(rJ, mem_off(t0 + 4 * g), (t0 + 4 * g) * row4);
    wave_sync();                                      // earlier reads of the stages are done
    if (mvalid) {
#pragma unroll
      for (int g = 0; g < G; ++g) *(u32x4 *)&stage[w][g][mslot] = raw[g];
    }
    wave_sync();
    float j[SEG], e = 0.f;
#pragma unroll
    for (int k = 0; k < SEG; ++k) {
      j[k] = __uint_as_float(stage[w][k >> 2][(k & 3) * 64 + slot]);
      e = beta * e + j[k];
    }
    x_e[par][w][lane] = e;
    __syncthreads();
    float cst = y_in, y = 0.f;
#pragma unroll
    for (int v = 0; v < NW; ++v) {
      if (v == w) y = cst;
      cst = bseg * cst + x_e[par][v][lane];
    }
    y_in = cst;
    uint32_t out[SEG];
#pragma unroll
    for (int k = 0; k < SEG; ++k) {
      y = beta * y + j[k];
      out[k] = __float_as_uint(y);
      if (INTEGRAL) { if (t0 + k < T) ysum += y; }
      else if (t0 + k < T && y > best) { best = y; tb = t0 + k; }
    }
    wave_sync();
    if (staged) {
#pragma unroll
      for (int k = 0; k < SEG; ++k) stage[w][k >> 2][(k & 3) * 64 + slot] = out[k];
    }
    wave_sync();
#pragma unroll
    for (int g = 0; g < G; ++g)
      st_b128(rY, mem_off(t0 + 4 * g), (t0 + 4 * g) * row4, *(const u32x4 *)&stage[w][g][mslot]);
  }

  // first maximiser over all segments (or, for the integral loss, the sum of the segments'
  // sums, added in wavefront order)
  x_best[w][lane] = INTEGRAL ? ysum : best;
  x_tb[w][lane] = tb;
  __syncthreads();
  best = x_best[0][lane];
  tb = x_tb[0][lane];
#pragma unroll
  for (int v = 1; v < NW; ++v) {
    const float bv = x_best[v][lane];
    const int tv = x_tb[v][lane];
    if (INTEGRAL) best += bv;
    else if (bv > best || (bv == best && tv < tb)) { best = bv; tb = tv; }
  }
  if (live && w == 0) { z[p] = best; tstar[p] = tb; }

  // softmax cross-entropy per sample (every wavefront, for dz)
  float m = live ? best : -INFINITY;
#pragma unroll
  for (int o = CW / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  const float ex = live ? expf(best - m) : 0.f;
  float sum = ex;
#pragma unroll
  for (int o = CW / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  int lab = lab_in;
  if (lab < 0 || lab >= C) { if (c == 0 && w == 0) atomicOr(err, 1); lab = 0; }
  float zl = (live && c == lab) ? best : 0.f;          // z[label], gathered across the group
#pragma unroll
  for (int o = CW / 2; o > 0; o >>= 1) zl += __shfl_xor(zl, o);
  const float d = live ? (ex / sum - (c == lab ? 1.f : 0.f)) / (float)B : 0.f;
  if (w == 0) {
    if (live) dz[p] = d;
    if (b < B && c == 0) loss_b[b] = m + logf(sum) - zl;
  }

  // dJ
  const float l2b = log2f(beta);
  for (int sb0 = 0; sb0 < T; sb0 += SB) {
    const int t0 = sb0 + SEG * w;
    float h;
    if (INTEGRAL) {
      // dz enters at every step: h_t = dz (1 - beta^(T-t)) / (1 - beta) at the segment's upper edge
      const int n = T - (t0 + SEG);
      h = n <= 0 ? 0.f : beta == 1.f ? d * (float)n : d * (1.f - exp2f((float)n * l2b)) / (1.f - beta);
    } else {
      const int n = tb - (t0 + SEG);                  // steps from the segment's upper edge up to t*
      h = n > 0 ? d * exp2f((float)n * l2b) : n == 0 ? d : 0.f;
    }
    uint32_t out[SEG];
#pragma unroll
    for (int k = SEG - 1; k >= 0; --k) {
      h = beta * h + ((INTEGRAL ? t0 + k < T : t0 + k == tb) ? d : 0.f);
      out[k] = HL ? pack_hl(h) : __float_as_uint(h);
    }
    wave_sync();
    if (staged) {
#pragma unroll
      for (int k = 0; k < SEG; ++k) stage[w][k >> 2][(k & 3) * 64 + slot] = out[k];
    }
    wave_sync();
#pragma unroll
    for (int g = 0; g < G; ++g)
      st_b128(rdJ, mem_off(t0 + 4 * g), (t0 + 4 * g) * row4, *(const u32x4 *)&stage[w][g][mslot]);
  }
}

// Readout reverse: h_t = beta h_{t+1} + dz [t == t*]; dJ_t = h_t.
template <bool HL>
__global__ __launch_bounds__(256) void readout_reverse_kernel(const float *__restrict__ dz, const int *__restrict__ tstar,
                                                              uint32_t *__restrict__ dJ, int T, int stride,
                                                              const float *__restrict__ beta_v, int ld, int integral) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= stride) return;
  const float beta = beta_v[p % ld];
  const float d = dz[p];
  const int ts = tstar[p];
  float h = 0.f;
  for (int t = T - 1; t >= 0; --t) {
    h = beta * h + (integral || t == ts ? d : 0.f);     // integral loss: every step feeds dz in
    dJ[(size_t)t * stride + p] = HL ? pack_hl(h) : __float_as_uint(h);
  }
}

// Gradient of the readout decays, per chain: y_t = beta y_{t-1} + J_t gives
// dL/dbeta = sum_{t >= 1} h_t y_{t-1} with h_t = dJ_t.  Summed over the batch by the reduction
// launch.  Only run when the decays are trained.
template <bool HL>
__global__ __launch_bounds__(256) void readout_beta_grad_kernel(const uint32_t *__restrict__ dJ, const float *__restrict__ Y,
                                                                float *__restrict__ db_part, int T, int stride) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= stride) return;
  float acc = 0.f;
#pragma unroll 4
  for (int t = 1; t < T; ++t) {
    const uint32_t w = dJ[(size_t)t * stride + p];
    const float h = HL ? bf16_value(w & 0xFFFFu) + bf16_value(w >> 16) : __uint_as_float(w);
    acc += h * Y[(size_t)(t - 1) * stride + p];
  }
  db_part[p] = acc;
}

#define SNN_MAX_JOBS 24
// beta <- clip(beta - lr dbeta, 0, 1) for several layers in one launch (the clip of the LIF listing).
struct BetaJobs {
  int njobs;
  int first[SNN_MAX_JOBS + 1];
  float *beta[SNN_MAX_JOBS];
  const float *dbeta[SNN_MAX_JOBS];
};
__global__ __launch_bounds__(256) void beta_update_kernel(const BetaJobs jobs, float lr) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= jobs.first[jobs.njobs]) return;
  int j = 0;
  while (j + 1 < jobs.njobs && i >= jobs.first[j + 1]) ++j;
  const int k = i - jobs.first[j];
  jobs.beta[j][k] = fminf(1.f, fmaxf(0.f, jobs.beta[j][k] - lr * jobs.dbeta[j][k]));
}

// ---------------------------------------------------------------- small utilities
// One wavefront that returns once `ticks` of the constant-rate device clock have passed (or
// after a bounded number of polls): a kernel of known duration for calibrating event timers.
__global__ __launch_bounds__(64) void wait_ticks_kernel(long long ticks, long long *__restrict__ out) {
  const long long t0 = wall_clock64();
  long long t = t0;
  for (int i = 0; i < (1 << 20) && t - t0 < ticks; ++i) t = wall_clock64();
  if (threadIdx.x == 0) out[0] = t - t0;
}

// dst[m][0..ld) = src[m][0..n) followed by zeros (input rasters whose rows are not 4-byte multiples).
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst,
                                                       long long rows, int n, int ld) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * ld) return;
  const long long r = i / ld;
  const int k = (int)(i - r * ld);
  dst[i] = k < n ? src[r * n + k] : 0;
}

// Input raster packed along time as numpy.packbits(x, axis=0) writes it (Section 2.1.4: eight
// spikes per byte, first step in the most significant bit): src [ceil(T/8)][B][n] -> dst
// [T][B][ld] bytes 0/1.  One thread per packed byte.
__global__ __launch_bounds__(256) void unpack_time_bits_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst,
                                                               int T, int B, int n, int ld) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long per_step = (long long)B * n;
  if (i >= (long long)((T + 7) / 8) * per_step) return;
  const int tp = (int)(i / per_step);
  const long long r = i - tp * per_step;
  const int b = (int)(r / n), k = (int)(r - (long long)b * n);
  const uint32_t bits = src[i];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int t = 8 * tp + j;
    if (t < T) dst[((long long)t * B + b) * ld + k] = (uint8_t)((bits >> (7 - j)) & 1u);
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *__restrict__ p, long long n_dwords) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_dwords) p[i] = 0u;
}

// Sum of the per-split partial results of the weight-gradient products, several matrices per
// launch.  out[i] = sum over splits of part[s][i].  A workgroup owns 256 consecutive floats
// of one job; its four wavefronts each add every fourth split (16-byte loads, eight in
// flight) and the four sums are combined through LDS in a fixed order, so the result does
// not depend on timing.  Tails that are not a multiple of four floats are done one by one.
// (Up to three reductions per layer: dW, dR and, with trained decays, the per-sample parts of dbeta.)
#define SNN_MAX_REDUCE_JOBS 36
struct ReduceJobs {
  int njobs;
  int first_block[SNN_MAX_REDUCE_JOBS + 1];
  const float *part[SNN_MAX_REDUCE_JOBS];
  float *out[SNN_MAX_REDUCE_JOBS];
  int splits[SNN_MAX_REDUCE_JOBS];
  long long n[SNN_MAX_REDUCE_JOBS];   // elements per matrix = stride between splits
};

// Mean of the per-sample losses in a fixed order, by one workgroup of 256 threads.
__device__ __forceinline__ void loss_mean_block(const float *__restrict__ loss_b, float *__restrict__ loss, int B,
                                                float *part) {
  float s = 0.f;
  for (int b = threadIdx.x; b < B; b += 256) s += loss_b[b];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = part[0] / (float)B;
}

__global__ __launch_bounds__(256) void loss_mean_kernel(const float *__restrict__ loss_b, float *__restrict__ loss, int B) {
  __shared__ float part[256];
  loss_mean_block(loss_b, loss, B, part);
}

// One workgroup beyond the last job (only launched when loss_b != NULL) takes the mean loss.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const ReduceJobs jobs, const float *__restrict__ loss_b,
                                                              float *__restrict__ loss, int B) {
  __shared__ float4 sm[4][64];
  if ((int)blockIdx.x >= jobs.first_block[jobs.njobs]) {
    loss_mean_block(loss_b, loss, B, (float *)sm);
    return;
  }
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first_block[j + 1]) ++j;
  const float *__restrict__ part = jobs.part[j];
  float *__restrict__ out = jobs.out[j];
  const int splits = jobs.splits[j];
  const long long n = jobs.n[j];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const long long i = ((long long)(blockIdx.x - jobs.first_block[j]) * 64 + lane) * 4;
  const bool vec = (n & 3) == 0;                      // every split slice is 16-byte aligned
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n) {
    const float *p = part + i;
    if (vec) {
      int k = w;
      for (; k + 28 < splits; k += 32) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *(const float4 *)(p + (size_t)(k + 4 * u) * n);
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
      }
      for (; k < splits; k += 4) {
        const float4 v = *(const float4 *)(p + (size_t)k * n);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    } else {
      for (int k = w; k < splits; k += 4) {
        const float *q = p + (size_t)k * n;
        acc.x += q[0];
        if (i + 1 < n) acc.y += q[1];
        if (i + 2 < n) acc.z += q[2];
        if (i + 3 < n) acc.w += q[3];
      }
    }
  }
  sm[w][lane] = acc;
  __syncthreads();
  if (w == 0 && i < n) {
    float4 r = sm[0][lane];
#pragma unroll
    for (int q = 1; q < 4; ++q) { r.x += sm[q][lane].x; r.y += sm[q][lane].y; r.z += sm[q][lane].z; r.w += sm[q][lane].w; }
    if (vec) {
      *(float4 *)(out + i) = r;
    } else {
      out[i] = r.x;
      if (i + 1 < n) out[i + 1] = r.y;
      if (i + 2 < n) out[i + 2] = r.z;
      if (i + 3 < n) out[i + 3] = r.w;
    }
  }
}

// Parameter update and operand refresh, several matrices W [K][N] (row-major) per launch:
//   W <- W - lr dW            (skipped when dW == NULL)
//   Qb[p][k][n] = piece_p(W[k][n])     contraction over n   (skipped when Qb == NULL)
//   Qf[p][n][k] = piece_p(W[k][n])     contraction over k   (32x32 tiles transposed in LDS)
struct ParamJobs {
  int njobs;
  int first_block[SNN_MAX_JOBS + 1];
  int blocks_x[SNN_MAX_JOBS];
  float *W[SNN_MAX_JOBS];
  const float *dW[SNN_MAX_JOBS];
  int K[SNN_MAX_JOBS], N[SNN_MAX_JOBS];
  uint16_t *Qf[SNN_MAX_JOBS];
  uint16_t *Qb[SNN_MAX_JOBS];
  int ldqf[SNN_MAX_JOBS], ldqb[SNN_MAX_JOBS];
  long long qf_plane[SNN_MAX_JOBS], qb_plane[SNN_MAX_JOBS];
};

__global__ __launch_bounds__(256) void param_update_kernel(const ParamJobs jobs, float lr, int nplanes) {
  __shared__ uint16_t tile[3][32][33];
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first_block[j + 1]) ++j;
  const int blk = blockIdx.x - jobs.first_block[j];
  float *__restrict__ W = jobs.W[j];
  const float *__restrict__ dW = jobs.dW[j];
  const int K = jobs.K[j], N = jobs.N[j];
  uint16_t *__restrict__ Qf = jobs.Qf[j];
  uint16_t *__restrict__ Qb = jobs.Qb[j];
  const int ldqf = jobs.ldqf[j], ldqb = jobs.ldqb[j];
  const long long qf_plane = jobs.qf_plane[j], qb_plane = jobs.qb_plane[j];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int n0 = (blk % jobs.blocks_x[j]) * 32, k0 = (blk / jobs.blocks_x[j]) * 32;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int k = k0 + ty + 8 * r, n = n0 + tx;
    float w = 0.f;
    if (k < K && n < N) {
      w = W[(size_t)k * N + n];
      if (dW) { w -= lr * dW[(size_t)k * N + n]; W[(size_t)k * N + n] = w; }
    }
    for (int p = 0; p < nplanes; ++p) {
      const uint16_t bits = (uint16_t)bf16_piece(w, p);
      tile[p][ty + 8 * r][tx] = bits;
      if (Qb && k < K && n < N) Qb[(size_t)p * qb_plane + (size_t)k * ldqb + n] = bits;
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int n = n0 + ty + 8 * r, k = k0 + tx;
    if (k < K && n < N)
      for (int p = 0; p < nplanes; ++p) Qf[(size_t)p * qf_plane + (size_t)n * ldqf + k] = tile[p][tx][ty + 8 * r];
  }
}

// Reduction of the per-split partial weight gradients and the parameter update in one launch,
// for the step that goes straight from snn_backward to snn_sgd_step: per matrix W [K][N],
//   dW = sum over the splits, in the order reduce_partials_kernel adds them (four interleaved
//        running sums, then ((s0 + s1) + s2) + s3): the same bits as the separate launch;
//   W <- W - lr dW, Qb and Qf refreshed as param_update_kernel does.
// A workgroup owns 8 rows x 32 columns (432 workgroups at 700-128-128-20, where 32 x 32 tiles
// would leave 108 to pull 28 MB of partial sums); every load of a partial is a full 128-byte
// row piece; the transposed operand leaves through LDS as 16 bytes per column (8 rows).
// One workgroup beyond the last job takes the mean loss when loss_b != NULL.
struct ReduceUpdateJobs {
  int njobs;
  int first_block[SNN_MAX_JOBS + 1];
  int blocks_x[SNN_MAX_JOBS];
  float *W[SNN_MAX_JOBS], *dW[SNN_MAX_JOBS];
  const float *part[SNN_MAX_JOBS];     // NULL: dW holds the gradient already (a single split)
  int splits[SNN_MAX_JOBS];
  int K[SNN_MAX_JOBS], N[SNN_MAX_JOBS];
  uint16_t *Qf[SNN_MAX_JOBS];
  uint16_t *Qb[SNN_MAX_JOBS];
  int ldqf[SNN_MAX_JOBS], ldqb[SNN_MAX_JOBS];
  long long qf_plane[SNN_MAX_JOBS], qb_plane[SNN_MAX_JOBS];
};

__global__ __launch_bounds__(256) void reduce_update_kernel(const ReduceUpdateJobs jobs, float lr, int nplanes,
                                                            const float *__restrict__ loss_b, float *__restrict__ loss,
                                                            int B) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[3][32][8];
  __shared__ float lsum[256];
  if ((int)blockIdx.x >= jobs.first_block[jobs.njobs]) {
    loss_mean_block(loss_b, loss, B, lsum);
    return;
  }
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first_block[j + 1]) ++j;
  const int blk = blockIdx.x - jobs.first_block[j];
  float *__restrict__ W = jobs.W[j];
  float *__restrict__ dW = jobs.dW[j];
  const float *__restrict__ part = jobs.part[j];
  const int splits = jobs.splits[j];
  const int K = jobs.K[j], N = jobs.N[j];
  uint16_t *__restrict__ Qf = jobs.Qf[j];
  uint16_t *__restrict__ Qb = jobs.Qb[j];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int n0 = (blk % jobs.blocks_x[j]) * 32, k0 = (blk / jobs.blocks_x[j]) * 8;
  const int k = k0 + ty, n = n0 + tx;
  float w = 0.f;
  if (k < K && n < N) {
    const size_t idx = (size_t)k * N + n, kn = (size_t)K * N;
    float g;
    if (part) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      int s = 0;
      // (all loads of a round are in flight before the first sum: the kernel is a few memory round
      // trips long, and 32 splits are one round instead of four)
      for (; s + 32 <= splits; s += 32) {
        float v[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) v[u] = part[(size_t)(s + u) * kn + idx];
#pragma unroll
        for (int u = 0; u < 32; ++u) acc[u & 3] += v[u];
      }
      for (; s + 8 <= splits; s += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(s + u) * kn + idx];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u & 3] += v[u];
      }
      for (; s < splits; ++s) acc[s & 3] += part[(size_t)s * kn + idx];
      g = ((acc[0] + acc[1]) + acc[2]) + acc[3];
      dW[idx] = g;
    } else {
      g = dW[idx];
    }
    w = W[idx] - lr * g;
    W[idx] = w;
  }
  for (int p = 0; p < nplanes; ++p) {
    const uint16_t bits = (uint16_t)bf16_piece(w, p);
    tile[p][tx][ty] = bits;
    if (Qb && k < K && n < N) Qb[(size_t)p * jobs.qb_plane[j] + (size_t)k * jobs.ldqb[j] + n] = bits;
  }
  __syncthreads();
  // Qf[p][n][k0 .. k0+7]: rows beyond K are zeros, as the padding of Qf is
  if ((int)threadIdx.x < 32 * nplanes) {
    const int p = threadIdx.x >> 5, nn = n0 + tx;
    if (nn < N) *(uint4 *)&Qf[(size_t)p * jobs.qf_plane[j] + (size_t)nn * jobs.ldqf[j] + k0] = *(const uint4 *)&tile[p][tx][0];
  }
}

}  // namespace snn
