// MFMA matrix products of the training step, gfx950.
//
// One kernel template computes C[i][j] = sum_k P(i,k) * Q(j,k) with bfloat16 operands and
// fp32 accumulation on v_mfma_f32_32x32x16_bf16.  What differs between the products of the
// path is only how the operand tiles reach LDS:
//
//   direct      the contraction index is the fastest axis in memory
//                 current product   I = S W          P = S [m][k] (0/1 bytes)  Q = W^T planes
//                 input gradient    dS = dI W^T      P = dI [m][n]             Q = W planes
//   transposed  the contraction index is the slowest axis (contraction over the T*B rows)
//                 weight gradient   dW = S^T dI      P = S [m][i] (0/1 bytes)  Q = dI [m][j]
//               8x4 / 8x2 element blocks are transposed in registers on their way to LDS.
//
// "Planes": a real operand enters as bfloat16 pieces of the split x = hi + mid + lo.
//   weights            pre-split in memory: one plane when rounded to bfloat16, three for
//                      fp32 products
//   current gradients  with rounded weights: one dword per element holding hi (low half) and
//                      lo (high half), written that way by the reverse scans ("HL");
//                      with fp32 products: plain fp32, split in three on the way to LDS
// An LDS stage holds every plane of both operand tiles and the MFMA loop runs over the plane
// pairs (p, q) with p + q < max(#P planes, #Q planes): all pairs whose product is above
// 2^-24 relative.  0/1 operands have a single, exact plane.
//
// Epilogues: plain store (optionally one partial result per contraction split), or one step
// of a recurrent LIF layer, forward or reverse, applied to the recurrent product.
#pragma once
#include "common.cuh"

namespace snn {

enum { P_U8 = 0, P_HL = 1, P_F32S = 2, P_T_U8 = 3 };
enum { Q_BF16 = 0, Q_T_HL = 1, Q_T_F32S = 2 };
enum { EPI_STORE = 0, EPI_RLIF_FWD = 1, EPI_RLIF_REV = 2 };

struct GemmArgs {
  const void *P;
  const void *Q;
  float *C;
  int rows, cols;            // extent of C
  int kc;                    // contraction length (elements that may be read along k)
  int ldp, ldq, ldc;         // leading dimensions in elements
  int p_align;               // P_U8 / P_T_U8: widest aligned load allowed (8, 4 or 1 bytes)
  int p_ivalid;              // P_T_U8: number of valid columns of P (rows of C)
  long long q_plane_stride;  // Q_BF16: elements between planes
  int kc_per_split;          // contraction range per blockIdx.y (multiple of 64)
  long long c_split_stride;  // elements between partial results
  int tiles_m, tiles_n;
  // recurrent-step epilogues (rows = B, cols = N, all [B][ld] with ld = ldc)
  const float *e_cur;        // fwd: I_t            rev: dS_t
  const float *e_v;          // fwd: V_t            rev: V_t
  const uint8_t *e_s;        // fwd: S_t
  const float *e_g;          // rev: g (dL/dV_{t+1}), fp32
  float *e_out_f;            // fwd: V_{t+1}        rev: new g
  uint8_t *e_out_s;          // fwd: S_{t+1}
  uint32_t *e_out_di;        // rev: dI_{t-1} (NULL at t = 0), fp32 bits or HL
  int e_di_hl;
  float beta, theta, slope;
  int surrogate;
};

__device__ __forceinline__ float surrogate_eval(int kind, float k, float x) {
  switch (kind) {
    case 0: { float d = 1.0f + k * fabsf(x); return 1.0f / (d * d); }
    case 1: { float u = 1.5707963267948966f * k * x; return (0.5f * k) / (1.0f + u * u); }
    case 2: { float s = 1.0f / (1.0f + __expf(-k * x)); return k * s * (1.0f - s); }
    default: return fmaxf(0.0f, 1.0f - fabsf(k * x));
  }
}

// ------------------------------------------------------------------ operand loaders
// Each loader keeps one tile's worth of raw global data in registers (load) and later
// converts and writes all its planes to LDS (store), so global latency overlaps the MFMAs.
// `tile` points at plane 0; plane p starts ROWS*128 bytes further.

template <int MODE, int ROWS> struct LoaderP;

template <int ROWS> struct LoaderP<P_U8, ROWS> {
  static constexpr int PLANES = 1;
  static constexpr int CH = (ROWS * 8 + 255) / 256;
  uint32_t raw[CH][2];
  __device__ __forceinline__ void load(const GemmArgs &a, int row0, int k0, int kend, int tid) {
    const uint8_t *P = (const uint8_t *)a.P;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      int cid = tid + 256 * c;
      int r = cid >> 3, ch = cid & 7;
      int grow = row0 + r, k = k0 + ch * 8;
      uint32_t lo = 0, hi = 0;
      if (cid < ROWS * 8 && grow < a.rows && k < kend) {
        const uint8_t *p = P + (size_t)grow * a.ldp + k;
        if (a.p_align == 8) {
          uint2 v = *(const uint2 *)p; lo = v.x; hi = v.y;
        } else if (a.p_align == 4) {
          lo = *(const uint32_t *)p;
          if (k + 4 < kend) hi = *(const uint32_t *)(p + 4);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (k + e < kend) lo |= (uint32_t)p[e] << (8 * e);
            if (k + 4 + e < kend) hi |= (uint32_t)p[4 + e] << (8 * e);
          }
        }
      }
      raw[c][0] = lo; raw[c][1] = hi;
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      int cid = tid + 256 * c;
      if (cid < ROWS * 8) {
        uint4 d;
        d.x = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][0], 0x0C010C00u));
        d.y = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][0], 0x0C030C02u));
        d.z = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][1], 0x0C010C00u));
        d.w = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][1], 0x0C030C02u));
        *(uint4 *)(tile + tile_off(cid >> 3, cid & 7)) = d;
      }
    }
  }
};

// P[m][k] dwords, each holding hi (bits 0..15) and lo (bits 16..31) of one value.
template <int ROWS> struct LoaderP<P_HL, ROWS> {
  static constexpr int PLANES = 2;
  static constexpr int CH = (ROWS * 8 + 255) / 256;
  uint4 raw[CH][2];
  __device__ __forceinline__ void load(const GemmArgs &a, int row0, int k0, int kend, int tid) {
    const uint32_t *P = (const uint32_t *)a.P;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      int cid = tid + 256 * c;
      int r = cid >> 3, ch = cid & 7;
      int grow = row0 + r, k = k0 + ch * 8;
      uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
      if (cid < ROWS * 8 && grow < a.rows && k < kend) {
        const uint4 *p = (const uint4 *)(P + (size_t)grow * a.ldp + k);
        v0 = p[0]; v1 = p[1];
      }
      raw[c][0] = v0; raw[c][1] = v1;
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      int cid = tid + 256 * c;
      if (cid < ROWS * 8) {
        const int off = tile_off(cid >> 3, cid & 7);
        uint4 h, l;
        h.x = __builtin_amdgcn_perm(raw[c][0].y, raw[c][0].x, 0x05040100u);
        h.y = __builtin_amdgcn_perm(raw[c][0].w, raw[c][0].z, 0x05040100u);
        h.z = __builtin_amdgcn_perm(raw[c][1].y, raw[c][1].x, 0x05040100u);
        h.w = __builtin_amdgcn_perm(raw[c][1].w, raw[c][1].z, 0x05040100u);
        l.x = __builtin_amdgcn_perm(raw[c][0].y, raw[c][0].x, 0x07060302u);
        l.y = __builtin_amdgcn_perm(raw[c][0].w, raw[c][0].z, 0x07060302u);
        l.z = __builtin_amdgcn_perm(raw[c][1].y, raw[c][1].x, 0x07060302u);
        l.w = __builtin_amdgcn_perm(raw[c][1].w, raw[c][1].z, 0x07060302u);
        *(uint4 *)(tile + off) = h;
        *(uint4 *)(tile + ROWS * 128 + off) = l;
      }
    }
  }
};

template <int ROWS> struct LoaderP<P_F32S, ROWS> {
  static constexpr int PLANES = 3;
  static constexpr int CH = (ROWS * 8 + 255) / 256;
  float4 raw[CH][2];
  __device__ __forceinline__ void load(const GemmArgs &a, int row0, int k0, int kend, int tid) {
    const float *P = (const float *)a.P;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      int cid = tid + 256 * c;
      int r = cid >> 3, ch = cid & 7;
      int grow = row0 + r, k = k0 + ch * 8;
      float4 v0 = make_float4(0, 0, 0, 0), v1 = v0;
      if (cid < ROWS * 8 && grow < a.rows && k < kend) {
        const float4 *p = (const float4 *)(P + (size_t)grow * a.ldp + k);
        v0 = p[0]; v1 = p[1];
      }
      raw[c][0] = v0; raw[c][1] = v1;
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      int cid = tid + 256 * c;
      if (cid < ROWS * 8) {
        const int off = tile_off(cid >> 3, cid & 7);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
          uint4 d;
          d.x = pack2(bf16_piece(raw[c][0].x, pl), bf16_piece(raw[c][0].y, pl));
          d.y = pack2(bf16_piece(raw[c][0].z, pl), bf16_piece(raw[c][0].w, pl));
          d.z = pack2(bf16_piece(raw[c][1].x, pl), bf16_piece(raw[c][1].y, pl));
          d.w = pack2(bf16_piece(raw[c][1].z, pl), bf16_piece(raw[c][1].w, pl));
          *(uint4 *)(tile + pl * ROWS * 128 + off) = d;
        }
      }
    }
  }
};

// P[m][i] bytes, contraction index m slowest.  One unit = 8 consecutive m x 4 consecutive i.
template <int ROWS> struct LoaderP<P_T_U8, ROWS> {
  static constexpr int PLANES = 1;
  static constexpr int UNITS = ROWS * 2;                  // (ROWS/4) column groups x 8 m groups
  static constexpr int UP = (UNITS + 255) / 256;
  uint32_t raw[UP][8];
  __device__ __forceinline__ void load(const GemmArgs &a, int row0, int k0, int kend, int tid) {
    const uint8_t *P = (const uint8_t *)a.P;
#pragma unroll
    for (int c = 0; c < UP; ++c) {
      int u = tid + 256 * c;
      int ig = u % (ROWS / 4), mg = u / (ROWS / 4);
      int i = row0 + 4 * ig;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        int m = k0 + 8 * mg + r;
        uint32_t v = 0;
        if (u < UNITS && m < kend && i < a.p_ivalid) {
          const uint8_t *p = P + (size_t)m * a.ldp + i;
          if (a.p_align >= 4) {
            v = *(const uint32_t *)p;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (i + e < a.p_ivalid) v |= (uint32_t)p[e] << (8 * e);
          }
        }
        raw[c][r] = v;
      }
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < UP; ++c) {
      int u = tid + 256 * c;
      if (u < UNITS) {
        int ig = u % (ROWS / 4), mg = u / (ROWS / 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // byte e of raw[2h] -> bits 0..7, byte e of raw[2h+1] -> bits 16..23
          const uint32_t sel = 0x0C000C00u | ((4u + e) << 16) | (uint32_t)e;
          uint4 d;
          d.x = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][1], raw[c][0], sel));
          d.y = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][3], raw[c][2], sel));
          d.z = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][5], raw[c][4], sel));
          d.w = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][7], raw[c][6], sel));
          *(uint4 *)(tile + tile_off(4 * ig + e, mg)) = d;
        }
      }
    }
  }
};

template <int MODE, int ROWS, int NPL> struct LoaderQ;

// Q[plane][j][k] bfloat16, allocated with rows padded to 128 and k padded to 64 (zeros).
template <int ROWS, int NPL> struct LoaderQ<Q_BF16, ROWS, NPL> {
  static constexpr int PLANES = NPL;
  static constexpr int CH = (ROWS * 8 + 255) / 256;
  uint4 raw[NPL][CH];
  __device__ __forceinline__ void load(const GemmArgs &a, int col0, int k0, int, int tid) {
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl) {
      const uint16_t *Q = (const uint16_t *)a.Q + (size_t)pl * a.q_plane_stride;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        int cid = tid + 256 * c;
        int r = cid >> 3, ch = cid & 7;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (cid < ROWS * 8) v = *(const uint4 *)(Q + (size_t)(col0 + r) * a.ldq + k0 + ch * 8);
        raw[pl][c] = v;
      }
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        int cid = tid + 256 * c;
        if (cid < ROWS * 8) *(uint4 *)(tile + pl * ROWS * 128 + tile_off(cid >> 3, cid & 7)) = raw[pl][c];
      }
  }
};

// Q[m][j] HL dwords, contraction index m slowest, ld a multiple of 8 with zero padding.
// One unit = 8 consecutive m x 2 consecutive j.
template <int ROWS, int NPL> struct LoaderQ<Q_T_HL, ROWS, NPL> {
  static_assert(NPL == 2, "hi and lo");
  static constexpr int PLANES = 2;
  static constexpr int UNITS = ROWS * 4;
  static constexpr int UQ = (UNITS + 255) / 256;
  uint2 raw[UQ][8];
  __device__ __forceinline__ void load(const GemmArgs &a, int col0, int k0, int kend, int tid) {
    const uint32_t *Q = (const uint32_t *)a.Q;
#pragma unroll
    for (int c = 0; c < UQ; ++c) {
      int u = tid + 256 * c;
      int jg = u % (ROWS / 2), mg = u / (ROWS / 2);
      int j = col0 + 2 * jg;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        int m = k0 + 8 * mg + r;
        uint2 v = make_uint2(0u, 0u);
        if (u < UNITS && m < kend && j < a.ldq) v = *(const uint2 *)(Q + (size_t)m * a.ldq + j);
        raw[c][r] = v;
      }
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < UQ; ++c) {
      int u = tid + 256 * c;
      if (u < UNITS) {
        int jg = u % (ROWS / 2), mg = u / (ROWS / 2);
        const int o0 = tile_off(2 * jg, mg), o1 = tile_off(2 * jg + 1, mg);
#pragma unroll
        for (int pl = 0; pl < 2; ++pl) {
          const uint32_t sel = pl == 0 ? 0x05040100u : 0x07060302u;
          uint4 d0, d1;
          d0.x = __builtin_amdgcn_perm(raw[c][1].x, raw[c][0].x, sel);
          d0.y = __builtin_amdgcn_perm(raw[c][3].x, raw[c][2].x, sel);
          d0.z = __builtin_amdgcn_perm(raw[c][5].x, raw[c][4].x, sel);
          d0.w = __builtin_amdgcn_perm(raw[c][7].x, raw[c][6].x, sel);
          d1.x = __builtin_amdgcn_perm(raw[c][1].y, raw[c][0].y, sel);
          d1.y = __builtin_amdgcn_perm(raw[c][3].y, raw[c][2].y, sel);
          d1.z = __builtin_amdgcn_perm(raw[c][5].y, raw[c][4].y, sel);
          d1.w = __builtin_amdgcn_perm(raw[c][7].y, raw[c][6].y, sel);
          *(uint4 *)(tile + pl * ROWS * 128 + o0) = d0;
          *(uint4 *)(tile + pl * ROWS * 128 + o1) = d1;
        }
      }
    }
  }
};

// Q[m][j] fp32, contraction index m slowest; split into three bfloat16 pieces on the way.
template <int ROWS, int NPL> struct LoaderQ<Q_T_F32S, ROWS, NPL> {
  static_assert(NPL == 3, "hi, mid and lo");
  static constexpr int PLANES = 3;
  static constexpr int UNITS = ROWS * 4;
  static constexpr int UQ = (UNITS + 255) / 256;
  float2 raw[UQ][8];
  __device__ __forceinline__ void load(const GemmArgs &a, int col0, int k0, int kend, int tid) {
    const float *Q = (const float *)a.Q;
#pragma unroll
    for (int c = 0; c < UQ; ++c) {
      int u = tid + 256 * c;
      int jg = u % (ROWS / 2), mg = u / (ROWS / 2);
      int j = col0 + 2 * jg;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        int m = k0 + 8 * mg + r;
        float2 v = make_float2(0.f, 0.f);
        if (u < UNITS && m < kend && j < a.ldq) v = *(const float2 *)(Q + (size_t)m * a.ldq + j);
        raw[c][r] = v;
      }
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < UQ; ++c) {
      int u = tid + 256 * c;
      if (u < UNITS) {
        int jg = u % (ROWS / 2), mg = u / (ROWS / 2);
        const int o0 = tile_off(2 * jg, mg), o1 = tile_off(2 * jg + 1, mg);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
          uint4 d0, d1;
          d0.x = pack2(bf16_piece(raw[c][0].x, pl), bf16_piece(raw[c][1].x, pl));
          d0.y = pack2(bf16_piece(raw[c][2].x, pl), bf16_piece(raw[c][3].x, pl));
          d0.z = pack2(bf16_piece(raw[c][4].x, pl), bf16_piece(raw[c][5].x, pl));
          d0.w = pack2(bf16_piece(raw[c][6].x, pl), bf16_piece(raw[c][7].x, pl));
          d1.x = pack2(bf16_piece(raw[c][0].y, pl), bf16_piece(raw[c][1].y, pl));
          d1.y = pack2(bf16_piece(raw[c][2].y, pl), bf16_piece(raw[c][3].y, pl));
          d1.z = pack2(bf16_piece(raw[c][4].y, pl), bf16_piece(raw[c][5].y, pl));
          d1.w = pack2(bf16_piece(raw[c][6].y, pl), bf16_piece(raw[c][7].y, pl));
          *(uint4 *)(tile + pl * ROWS * 128 + o0) = d0;
          *(uint4 *)(tile + pl * ROWS * 128 + o1) = d1;
        }
      }
    }
  }
};

// ------------------------------------------------------------------ the kernel
// 256 threads = WM x WN wavefronts, each owning TM x TN MFMA tiles of 32x32.  One LDS stage;
// the next tile's global loads are in flight while the MFMAs of the current one run.
template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs a) {
  static_assert(WM * WN == 4, "four wavefronts per workgroup");
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  typedef LoaderP<PM, BM> LP;
  typedef LoaderQ<QM, BN, NQP> LQ;
  constexpr int NPP = LP::PLANES;
  constexpr int NMAX = NPP > NQP ? NPP : NQP;
  constexpr int PT = BM * 128, QT = BN * 128;       // bytes of one plane of a tile
  static_assert(NPP * PT + NQP * QT <= 65536, "static LDS limit");
  __shared__ __attribute__((aligned(16))) char lds[NPP * PT + NQP * QT];
  char *const lds_q = lds + NPP * PT;

  // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // tiles (column tiles fastest) so that tiles sharing a row slab of P share an L2.
  const int ntiles = a.tiles_m * a.tiles_n;
  const int per_xcd = (ntiles + 7) >> 3;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= ntiles) return;
  const int row0 = (tile / a.tiles_n) * BM;
  const int col0 = (tile % a.tiles_n) * BN;
  const int kbeg = blockIdx.y * a.kc_per_split;
  const int kend = min(a.kc, kbeg + a.kc_per_split);
  const int nk = kend > kbeg ? (kend - kbeg + 63) >> 6 : 0;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  LP lp;
  LQ lq;
  if (nk > 0) {
    lp.load(a, row0, kbeg, kend, tid);
    lq.load(a, col0, kbeg, kend, tid);
    lp.store(lds, tid);
    lq.store(lds_q, tid);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) {
      lp.load(a, row0, kbeg + (kt + 1) * 64, kend, tid);
      lq.load(a, col0, kbeg + (kt + 1) * 64, kend, tid);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[NPP][TM], bq[NQP][TN];
      const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
      for (int p = 0; p < NPP; ++p)
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[p][i] = *(const bf16x8 *)(lds + p * PT + tile_off((wm * TM + i) * 32 + (lane & 31), chunk));
#pragma unroll
      for (int q = 0; q < NQP; ++q)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bq[q][j] = *(const bf16x8 *)(lds_q + q * QT + tile_off((wn * TN + j) * 32 + (lane & 31), chunk));
      // smallest products first
#pragma unroll
      for (int s = NMAX - 1; s >= 0; --s)
#pragma unroll
        for (int p = 0; p < NPP; ++p) {
          const int q = s - p;
          if (q >= 0 && q < NQP) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[p][i], bq[q][j], acc[i][j], 0, 0, 0);
          }
        }
    }
    if (more) {
      __syncthreads();
      lp.store(lds, tid);
      lq.store(lds_q, tid);
      __syncthreads();
    }
  }

  // Accumulator layout of the 32x32 MFMA: lane holds column (lane & 31); register r holds
  // row 8*(r/4) + 4*(lane/32) + (r%4).
  float *C = a.C + (size_t)blockIdx.y * a.c_split_stride;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = col0 + (wn * TN + j) * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < a.rows && col < a.cols) {
          const size_t o = (size_t)row * a.ldc + col;
          const float v = acc[i][j][r];
          if (EPI == EPI_STORE) {
            C[o] = v;
          } else if (EPI == EPI_RLIF_FWD) {
            // V_{t+1} = beta V_t + I_t + S_t R - theta S_t ; S_{t+1} = [V_{t+1} > theta]
            const float s = (float)a.e_s[o];
            const float vn = a.beta * a.e_v[o] + a.e_cur[o] + v - a.theta * s;
            a.e_out_f[o] = vn;
            a.e_out_s[o] = vn > a.theta ? 1 : 0;
          } else {
            // g_t = beta g_{t+1} + surr(V_t - theta) (dS_t - theta g_{t+1} + g_{t+1} R^T)
            const float g = a.e_g[o];
            const float q = a.e_cur[o] - a.theta * g + v;
            const float gn = a.beta * g + surrogate_eval(a.surrogate, a.slope, a.e_v[o] - a.theta) * q;
            a.e_out_f[o] = gn;
            if (a.e_out_di) a.e_out_di[o] = a.e_di_hl ? pack_hl(gn) : __float_as_uint(gn);
          }
        }
      }
    }
}

template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP>
static hipError_t gemm_launch(GemmArgs a, int splits, hipStream_t st) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  a.tiles_m = (a.rows + BM - 1) / BM;
  a.tiles_n = (a.cols + BN - 1) / BN;
  const int ntiles = a.tiles_m * a.tiles_n;
  const int per_xcd = (ntiles + 7) / 8;
  dim3 grid(per_xcd * 8, splits, 1);
  hipLaunchKernelGGL((gemm_kernel<PM, QM, EPI, WM, WN, TM, TN, NQP>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace snn
