// Time scans, readout, loss and parameter kernels of the training step, gfx950.
//
// The LIF scans are bound by HBM traffic: one thread owns VEC adjacent chains
// (b, n..n+VEC-1), keeps their state in registers for all T steps and streams the per-step
// rows.  Loads do not depend on the recurrence, so a block of U steps is fetched while the
// previous block is being integrated.
#pragma once
#include "common.cuh"

namespace snn {

template <int VEC> struct VecF;
template <> struct VecF<1> { typedef float type; };
template <> struct VecF<2> { typedef float2 type; };
template <> struct VecF<4> { typedef float4 type; };
template <int VEC> struct VecU;
template <> struct VecU<1> { typedef uint32_t type; };
template <> struct VecU<2> { typedef uint2 type; };
template <> struct VecU<4> { typedef uint4 type; };

template <int VEC> __device__ __forceinline__ void vload(float (&d)[VEC], const float *p) {
  typename VecF<VEC>::type v = *(const typename VecF<VEC>::type *)p;
  const float *f = (const float *)&v;
#pragma unroll
  for (int i = 0; i < VEC; ++i) d[i] = f[i];
}
template <int VEC> __device__ __forceinline__ void vstore(float *p, const float (&d)[VEC]) {
  typename VecF<VEC>::type v;
  float *f = (float *)&v;
#pragma unroll
  for (int i = 0; i < VEC; ++i) f[i] = d[i];
  *(typename VecF<VEC>::type *)p = v;
}
template <int VEC> __device__ __forceinline__ void vstore_u32(uint32_t *p, const uint32_t (&d)[VEC]) {
  typename VecU<VEC>::type v;
  uint32_t *f = (uint32_t *)&v;
#pragma unroll
  for (int i = 0; i < VEC; ++i) f[i] = d[i];
  *(typename VecU<VEC>::type *)p = v;
}
template <int VEC> __device__ __forceinline__ void vstore_u8(uint8_t *p, const uint32_t (&s)[VEC]) {
  if (VEC == 1) p[0] = (uint8_t)s[0];
  else if (VEC == 2) *(uint16_t *)p = (uint16_t)(s[0] | (s[1] << 8));
  else *(uint32_t *)p = s[0] | (s[1] << 8) | (s[2] << 16) | (s[3] << 24);
}

// ---------------------------------------------------------------- LIF forward (Eq. 1-2)
// S_t = [V_t > theta]; store V_t, S_t; V_{t+1} = beta V_t + I_t - theta S_t; V_0 = 0.
// `stride` = B * ld elements between time steps; threads cover the stride (padding
// columns included: their currents are zero, so they stay silent).
template <int VEC, int U>
__global__ __launch_bounds__(256) void lif_forward_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                          uint8_t *__restrict__ S, int T, long long stride,
                                                          float beta, float theta) {
  const long long p = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (p >= stride) return;
  I += p; V += p; S += p;
  float v[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) v[i] = 0.f;
  float a[U][VEC], b[U][VEC];

  auto fetch = [&](float (&buf)[U][VEC], int t0) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (t0 + u < T) vload<VEC>(buf[u], I + (long long)(t0 + u) * stride);
  };
  auto integrate = [&](float (&buf)[U][VEC], int t0) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (t0 + u < T) {
        uint32_t s[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) s[i] = v[i] > theta ? 1u : 0u;
        vstore<VEC>(V + (long long)(t0 + u) * stride, v);
        vstore_u8<VEC>(S + (long long)(t0 + u) * stride, s);
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = beta * v[i] + buf[u][i] - (s[i] ? theta : 0.f);
      }
  };
  fetch(a, 0);
  for (int t0 = 0; t0 < T; t0 += 2 * U) {
    fetch(b, t0 + U);
    integrate(a, t0);
    fetch(a, t0 + 2 * U);
    integrate(b, t0 + U);
  }
}

// ---------------------------------------------------------------- LIF reverse, fused surrogate
// g = 0; for t = T-1..0: dI_t = g; g = beta g + surr(V_t - theta) (dS_t - theta g).
// dI is written as fp32 or, when HL, in the hi/lo form the bfloat16 products read.
template <int SURR> __device__ __forceinline__ float surr(float k, float x) {
  if (SURR == 0) { float d = 1.0f + k * fabsf(x); return 1.0f / (d * d); }
  if (SURR == 1) { float u = 1.5707963267948966f * k * x; return (0.5f * k) / (1.0f + u * u); }
  if (SURR == 2) { float s = 1.0f / (1.0f + __expf(-k * x)); return k * s * (1.0f - s); }
  return fmaxf(0.0f, 1.0f - fabsf(k * x));
}

template <int VEC, int U, int SURR, bool HL>
__global__ __launch_bounds__(256) void lif_reverse_kernel(const float *__restrict__ dS, const float *__restrict__ V,
                                                          uint32_t *__restrict__ dI, int T, long long stride,
                                                          float beta, float theta, float slope) {
  const long long p = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (p >= stride) return;
  dS += p; V += p; dI += p;
  float g[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) g[i] = 0.f;
  float a_ds[U][VEC], a_v[U][VEC], b_ds[U][VEC], b_v[U][VEC];

  // a block covers steps thi, thi-1, .., thi-U+1
  auto fetch = [&](float (&bds)[U][VEC], float (&bv)[U][VEC], int thi) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (thi - u >= 0) {
        vload<VEC>(bds[u], dS + (long long)(thi - u) * stride);
        vload<VEC>(bv[u], V + (long long)(thi - u) * stride);
      }
  };
  auto integrate = [&](float (&bds)[U][VEC], float (&bv)[U][VEC], int thi) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (thi - u >= 0) {
        uint32_t w[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) w[i] = HL ? pack_hl(g[i]) : __float_as_uint(g[i]);
        vstore_u32<VEC>(dI + (long long)(thi - u) * stride, w);
#pragma unroll
        for (int i = 0; i < VEC; ++i)
          g[i] = beta * g[i] + surr<SURR>(slope, bv[u][i] - theta) * (bds[u][i] - theta * g[i]);
      }
  };
  fetch(a_ds, a_v, T - 1);
  for (int thi = T - 1; thi >= 0; thi -= 2 * U) {
    fetch(b_ds, b_v, thi - U);
    integrate(a_ds, a_v, thi);
    fetch(a_ds, a_v, thi - 2 * U);
    integrate(b_ds, b_v, thi - U);
  }
}

// ---------------------------------------------------------------- cooperative scans
// With few chains (B*N of the order of the number of SIMDs) one wavefront per 64 chains
// cannot keep enough loads in flight: a wavefront has at most 63 outstanding memory
// operations.  Here NW wavefronts share 64 chains.  Time is cut into rounds of NW*U steps;
// in a round wavefront w fetches steps [w*U, w*U+U) of the round (all NW*U rows in flight at
// once, the next round's already requested), then the wavefronts integrate their segments
// one after the other, handing the state on through LDS.  The serial part is a few
// instructions per step; the memory system sees NW times the parallelism.
template <int NW, int U>
__global__ __launch_bounds__(NW * 64) void lif_forward_coop_kernel(const float *__restrict__ I, float *__restrict__ V,
                                                                   uint8_t *__restrict__ S, int T, long long stride,
                                                                   float beta, float theta) {
  __shared__ float hand[64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const long long p0 = (long long)blockIdx.x * 64 + lane;
  const bool live = p0 < stride;
  const long long p = live ? p0 : 0;
  I += p; V += p; S += p;
  float a[U], b[U];
  auto fetch = [&](float (&buf)[U], int t0) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (t0 + u < T) buf[u] = I[(long long)(t0 + u) * stride];
  };
  auto turn = [&](float (&buf)[U], int t0) {
    for (int ww = 0; ww < NW; ++ww) {
      if (ww == w) {
        float v = hand[lane];
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (t0 + u < T) {
            const bool s = v > theta;
            if (live) {
              V[(long long)(t0 + u) * stride] = v;
              S[(long long)(t0 + u) * stride] = s ? 1 : 0;
            }
            v = beta * v + buf[u] - (s ? theta : 0.f);
          }
        hand[lane] = v;
      }
      lds_barrier();
    }
  };
  if (w == 0) hand[lane] = 0.f;                    // V_0 = 0
  fetch(a, w * U);
  lds_barrier();
  for (int r0 = 0; r0 < T; r0 += 2 * NW * U) {
    fetch(b, r0 + NW * U + w * U);
    turn(a, r0 + w * U);
    fetch(a, r0 + 2 * NW * U + w * U);
    turn(b, r0 + NW * U + w * U);
  }
}

template <int NW, int U, int SURR, bool HL>
__global__ __launch_bounds__(NW * 64) void lif_reverse_coop_kernel(const float *__restrict__ dS,
                                                                   const float *__restrict__ V,
                                                                   uint32_t *__restrict__ dI, int T, long long stride,
                                                                   float beta, float theta, float slope) {
  __shared__ float hand[64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const long long p0 = (long long)blockIdx.x * 64 + lane;
  const bool live = p0 < stride;
  const long long p = live ? p0 : 0;
  dS += p; V += p; dI += p;
  float a_ds[U], a_v[U], b_ds[U], b_v[U];
  // a segment covers steps thi, thi-1, .., thi-U+1
  auto fetch = [&](float (&bds)[U], float (&bv)[U], int thi) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (thi - u >= 0) {
        bds[u] = dS[(long long)(thi - u) * stride];
        bv[u] = V[(long long)(thi - u) * stride];
      }
  };
  auto turn = [&](float (&bds)[U], float (&bv)[U], int thi) {
    for (int ww = 0; ww < NW; ++ww) {
      if (ww == w) {
        float g = hand[lane];
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (thi - u >= 0) {
            if (live) dI[(long long)(thi - u) * stride] = HL ? pack_hl(g) : __float_as_uint(g);
            g = beta * g + surr<SURR>(slope, bv[u] - theta) * (bds[u] - theta * g);
          }
        hand[lane] = g;
      }
      lds_barrier();
    }
  };
  if (w == 0) hand[lane] = 0.f;                    // g_T = 0
  fetch(a_ds, a_v, T - 1 - w * U);
  lds_barrier();
  for (int r0 = T - 1; r0 >= 0; r0 -= 2 * NW * U) {
    fetch(b_ds, b_v, r0 - NW * U - w * U);
    turn(a_ds, a_v, r0 - w * U);
    fetch(a_ds, a_v, r0 - 2 * NW * U - w * U);
    turn(b_ds, b_v, r0 - NW * U - w * U);
  }
}

// ---------------------------------------------------------------- LI readout, max over time
// y_t = beta y_{t-1} + J_t, y_{-1} = 0; z = max_t y_t; t* = first maximiser.
__global__ __launch_bounds__(256) void readout_forward_kernel(const float *__restrict__ J, float *__restrict__ Y,
                                                              float *__restrict__ z, int *__restrict__ tstar,
                                                              int T, int stride, float beta) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= stride) return;
  float y = 0.f, best = -INFINITY;
  int tb = 0;
#pragma unroll 8
  for (int t = 0; t < T; ++t) {
    y = beta * y + J[(size_t)t * stride + p];
    Y[(size_t)t * stride + p] = y;
    if (y > best) { best = y; tb = t; }
  }
  z[p] = best;
  tstar[p] = tb;
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

// Mean of the per-sample losses in a fixed order (one workgroup).
__global__ __launch_bounds__(256) void loss_mean_kernel(const float *__restrict__ loss_b, float *__restrict__ loss, int B) {
  __shared__ float part[256];
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

// The three kernels above in one launch, for C <= 64.  A wavefront holds 64/CW samples, CW
// lanes each (CW = power of two >= C); a lane scans one (b, c) chain over time, then the
// softmax is reduced across the CW lanes of a sample.  Per-sample losses go to loss_b; the
// workgroup that takes the last ticket adds them up in index order, so the mean is the same
// on every run.
template <int CW>
__global__ __launch_bounds__(256) void readout_loss_kernel(const float *__restrict__ J, float *__restrict__ Y,
                                                           float *__restrict__ z, int *__restrict__ tstar,
                                                           const int *__restrict__ labels, float *__restrict__ loss_b,
                                                           float *__restrict__ dz, float *__restrict__ loss,
                                                           int *__restrict__ ticket, int *__restrict__ err, int T,
                                                           int B, int C, int ldc, float beta) {
  constexpr int SPB = 256 / CW;                       // samples per workgroup
  const int c = threadIdx.x % CW;
  const int b = blockIdx.x * SPB + threadIdx.x / CW;
  const bool live = b < B && c < C;
  const size_t stride = (size_t)B * ldc;
  const size_t p = live ? (size_t)b * ldc + c : 0;
  float y = 0.f, best = -INFINITY;
  int tb = 0;
  if (live) {
    int t = 0;
    for (; t + 8 <= T; t += 8) {
      float j[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) j[u] = J[(size_t)(t + u) * stride + p];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        y = beta * y + j[u];
        Y[(size_t)(t + u) * stride + p] = y;
        if (y > best) { best = y; tb = t + u; }
      }
    }
    for (; t < T; ++t) {
      y = beta * y + J[(size_t)t * stride + p];
      Y[(size_t)t * stride + p] = y;
      if (y > best) { best = y; tb = t; }
    }
    z[p] = best;
    tstar[p] = tb;
  }
  float m = live ? best : -INFINITY;
#pragma unroll
  for (int o = CW / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  const float e = live ? expf(best - m) : 0.f;
  float sum = e;
#pragma unroll
  for (int o = CW / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  int lab = b < B ? labels[b] : 0;
  if (lab < 0 || lab >= C) { if (c == 0) atomicOr(err, 1); lab = 0; }
  float zl = (live && c == lab) ? best : 0.f;          // z[label], gathered across the group
#pragma unroll
  for (int o = CW / 2; o > 0; o >>= 1) zl += __shfl_xor(zl, o);
  if (live) dz[p] = (e / sum - (c == lab ? 1.f : 0.f)) / (float)B;
  if (b < B && c == 0) loss_b[b] = m + logf(sum) - zl;

  __shared__ int last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) last = atomicAdd(ticket, 1) == (int)gridDim.x - 1;
  __syncthreads();
  if (last) {
    __threadfence();
    __shared__ float part[256];
    float s = 0.f;
    for (int i = threadIdx.x; i < B; i += 256) s += loss_b[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) { loss[0] = part[0] / (float)B; *ticket = 0; }
  }
}

// Readout reverse: h_t = beta h_{t+1} + dz [t == t*]; dJ_t = h_t.
template <bool HL>
__global__ __launch_bounds__(256) void readout_reverse_kernel(const float *__restrict__ dz, const int *__restrict__ tstar,
                                                              uint32_t *__restrict__ dJ, int T, int stride, float beta) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= stride) return;
  const float d = dz[p];
  const int ts = tstar[p];
  float h = 0.f;
  for (int t = T - 1; t >= 0; --t) {
    h = beta * h + (t == ts ? d : 0.f);
    dJ[(size_t)t * stride + p] = HL ? pack_hl(h) : __float_as_uint(h);
  }
}

// ---------------------------------------------------------------- small utilities
// dst[m][0..ld) = src[m][0..n) followed by zeros (input rasters whose rows are not 4-byte multiples).
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst,
                                                       long long rows, int n, int ld) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * ld) return;
  const long long r = i / ld;
  const int k = (int)(i - r * ld);
  dst[i] = k < n ? src[r * n + k] : 0;
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
#define SNN_MAX_JOBS 16
struct ReduceJobs {
  int njobs;
  int first_block[SNN_MAX_JOBS + 1];
  const float *part[SNN_MAX_JOBS];
  float *out[SNN_MAX_JOBS];
  int splits[SNN_MAX_JOBS];
  long long n[SNN_MAX_JOBS];          // elements per matrix = stride between splits
};

__global__ __launch_bounds__(256) void reduce_partials_kernel(const ReduceJobs jobs) {
  __shared__ float4 sm[4][64];
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

}  // namespace snn
