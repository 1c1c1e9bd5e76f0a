// Recurrent LIF layers: V_{t+1} = beta V_t + I_t + S_t R - theta S_t, with S_t the spikes
// just emitted from V_t (R is [from][to]).  Every step needs all N spikes of a sample from
// the step before, so time is walked on the host side of the stream: one launch per step,
// each a [B x N] x [N x N] MFMA product whose epilogue applies the LIF update (forward) or
// the surrogate-gradient recursion (reverse).  Stream order is the inter-step barrier.
#pragma once
#include "gemm.cuh"
#include "scan.cuh"

namespace snn {

static hipError_t fill_zero(hipStream_t st, void *p, size_t bytes) {
  const long long n = (long long)(bytes / 4);
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint32_t *)p, n);
  return hipGetLastError();
}

// I, V [T][B][ld] fp32, S [T][B][ld] bytes; QRf[plane][to][from] bfloat16.
static hipError_t rlif_forward(hipStream_t st, bool fp32, int T, int B, int N, int ld, const float *I, float *V,
                               uint8_t *S, const uint16_t *QRf, int ldqr, long long qr_plane, float beta,
                               float theta) {
  const size_t stride = (size_t)B * ld;
  hipError_t e;
  if ((e = fill_zero(st, V, stride * 4)) != hipSuccess) return e;     // V_0 = 0
  if ((e = fill_zero(st, S, stride)) != hipSuccess) return e;         // hence S_0 = 0
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.ldp = ld; a.kc = ld; a.p_bytes = (unsigned)stride;
  a.Q = QRf; a.ldq = ldqr; a.q_plane_stride = qr_plane; a.q_bytes = (unsigned)((fp32 ? 3 : 1) * qr_plane * 2);
  a.rows = B; a.cols = N; a.ldc = ld;
  a.kc_per_split = (ld + 63) / 64 * 64;
  a.beta = beta; a.theta = theta;
  for (int t = 0; t + 1 < T; ++t) {
    a.P = S + t * stride;
    a.e_cur = I + t * stride; a.e_v = V + t * stride; a.e_s = S + t * stride;
    a.e_out_f = V + (t + 1) * stride; a.e_out_s = S + (t + 1) * stride;
    if (fp32) e = gemm_launch<P_U8, Q_BF16, EPI_RLIF_FWD, 1, 4, 1, 1, 3, 1>(a, 1, st);
    else e = gemm_launch<P_U8, Q_BF16, EPI_RLIF_FWD, 1, 4, 1, 1, 1, 2>(a, 1, st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// dS, V [T][B][ld] fp32; dI [T][B][ld] dwords (fp32, or HL with rounded weights); g0, g1
// [B][ld] fp32 scratch for dL/dV_{t+1}; QRb[plane][from][to] bfloat16.
static hipError_t rlif_reverse(hipStream_t st, bool fp32, int T, int B, int N, int ld, const float *dS, const float *V,
                               uint32_t *dI, float *g0, float *g1, const uint16_t *QRb, int ldqr,
                               long long qr_plane, float beta, float theta, int surrogate, float slope) {
  const size_t stride = (size_t)B * ld;
  hipError_t e;
  if ((e = fill_zero(st, g0, stride * 4)) != hipSuccess) return e;                              // g_T = 0
  if ((e = fill_zero(st, dI + (size_t)(T - 1) * stride, stride * 4)) != hipSuccess) return e;   // dI_{T-1} = 0
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.ldp = ld; a.kc = ld; a.p_bytes = (unsigned)(stride * 4);
  a.Q = QRb; a.ldq = ldqr; a.q_plane_stride = qr_plane; a.q_bytes = (unsigned)((fp32 ? 3 : 1) * qr_plane * 2);
  a.rows = B; a.cols = N; a.ldc = ld;
  a.kc_per_split = (ld + 63) / 64 * 64;
  a.beta = beta; a.theta = theta; a.surrogate = surrogate; a.slope = slope;
  a.e_di_hl = fp32 ? 0 : 1;
  float *g[2] = {g0, g1};
  int cur = 0;
  for (int t = T - 1; t >= 0; --t) {
    a.P = dI + (size_t)t * stride;                            // dI_t = g_{t+1}
    a.e_cur = dS + t * stride; a.e_v = V + t * stride;
    a.e_g = g[cur]; a.e_out_f = g[cur ^ 1];
    a.e_out_di = t > 0 ? dI + (size_t)(t - 1) * stride : nullptr;
    if (fp32) e = gemm_launch<P_F32S, Q_BF16, EPI_RLIF_REV, 1, 4, 1, 1, 3, 1>(a, 1, st);
    else e = gemm_launch<P_HL, Q_BF16, EPI_RLIF_REV, 1, 4, 1, 1, 1, 2>(a, 1, st);
    if (e != hipSuccess) return e;
    cur ^= 1;
  }
  return hipSuccess;
}

}  // namespace snn
