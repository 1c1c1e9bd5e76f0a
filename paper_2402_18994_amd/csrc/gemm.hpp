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
//               With the input raster packed along time (Section 2.1.4: eight steps of a channel
//               per byte) the weight gradient of layer 1 walks the contraction in another order,
//               which a sum does not mind: a 64-wide tile is one packed row (eight steps) of eight
//               consecutive samples, so that a byte of P is exactly one 16-byte chunk of a tile row
//               (P_T_BITS) and the rows of dI follow the same order (Q_T_*_PK).
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
// Global loads are buffer loads: a per-lane byte offset computed once per workgroup, plus a
// scalar offset that walks the contraction, so the inner loop spends no vector ALU work on
// addresses.  A lane that must read nothing (row, column or contraction tail) is given an
// offset beyond the buffer's size, for which the hardware returns zero.
//
// Epilogues: plain store (optionally one partial result per contraction split), or one step
// of a recurrent LIF layer, forward or reverse, applied to the recurrent product.
#pragma once
#include "common.hpp"

namespace snn {

enum { P_U8 = 0, P_HL = 1, P_F32S = 2, P_T_U8 = 3, P_T_BITS = 4 };
enum { Q_BF16 = 0, Q_T_HL = 1, Q_T_F32S = 2, Q_T_HL_PK = 3, Q_T_F32S_PK = 4 };
enum { EPI_STORE = 0 };

struct GemmArgs {
  const void *P;
  const void *Q;
  float *C;
  unsigned p_bytes, q_bytes; // sizes of the P and Q buffers (reads beyond them return zero)
  int rows, cols;            // extent of C
  int kc;                    // contraction length (elements that may be read along k)
  int ldp, ldq, ldc;         // leading dimensions in elements
  int p_ivalid;              // P_T_U8: number of valid columns of P (rows of C)
  long long q_plane_stride;  // Q_BF16: elements between planes
  int kc_per_split;          // contraction range per split (multiple of 64)
  int splits;
  long long c_split_stride;  // elements between partial results
  int tiles_m, tiles_n;
  int nt_store;              // store C non-temporally (large results that a later kernel streams once)
  int packed;                // P_T_U8 jobs: P is the raster packed along time; contraction in packed order
  int pk_T, pk_B;            // time steps and batch of the packed raster (B a multiple of 8)
};

// ------------------------------------------------------------------ operand loaders
// setup(): per-lane byte offsets and LDS offsets, once per workgroup.
// load():  issue the global loads of the 64-wide contraction tile starting at k0 into
//          registers (raw).  `kend` is the end of this workgroup's contraction range.
// store(): convert and write all planes to LDS.  `tile` points at plane 0; plane p starts
//          ROWS*128 bytes further.

template <int MODE, int ROWS> struct LoaderP;

// P[row][k] bytes (0/1).
template <int ROWS> struct LoaderP<P_U8, ROWS> {
  static constexpr int PLANES = 1;
  static constexpr int CH = (ROWS * 8 + 255) / 256;
  int voff[CH], loff[CH], kch[CH];
  uint32_t raw[CH][2];
  __device__ __forceinline__ void setup(const GemmArgs &a, int row0, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int cid = tid + 256 * c;
      const int r = cid >> 3, ch = cid & 7;
      const bool ok = cid < ROWS * 8 && row0 + r < a.rows;
      voff[c] = ok ? (row0 + r) * a.ldp + ch * 8 : OOB;
      loff[c] = tile_off(r & (ROWS - 1), ch);
      kch[c] = ch * 8;
    }
  }
  // Rows are 4-byte aligned and kend is a multiple of 4 (the host pads the raster otherwise):
  // two dword loads per chunk, no branches, so the loads of several tiles can stay in flight.
  __device__ __forceinline__ void load(const GemmArgs &, rsrc_t rs, int k0, int kend) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int k = k0 + kch[c];
      raw[c][0] = ld_b32(rs, k >= kend ? OOB : voff[c], k0);
      raw[c][1] = ld_b32(rs, k + 4 >= kend ? OOB : voff[c] + 4, k0);
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      if (tid + 256 * c < ROWS * 8) {
        uint4 d;
        d.x = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][0], 0x0C010C00u));
        d.y = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][0], 0x0C030C02u));
        d.z = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][1], 0x0C010C00u));
        d.w = spikes2_to_bf16(__builtin_amdgcn_perm(0u, raw[c][1], 0x0C030C02u));
        *(uint4 *)(tile + loff[c]) = d;
      }
    }
  }
};

// P[row][k] dwords: HL words (two planes) or fp32 (three planes, split here).
template <int ROWS, bool HL> struct LoaderPWord {
  static constexpr int PLANES = HL ? 2 : 3;
  static constexpr int CH = (ROWS * 8 + 255) / 256;
  int voff[CH], loff[CH], kch[CH];
  u32x4 raw[CH][2];
  __device__ __forceinline__ void setup(const GemmArgs &a, int row0, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int cid = tid + 256 * c;
      const int r = cid >> 3, ch = cid & 7;
      const bool ok = cid < ROWS * 8 && row0 + r < a.rows;
      voff[c] = ok ? ((row0 + r) * a.ldp + ch * 8) * 4 : OOB;
      loff[c] = tile_off(r & (ROWS - 1), ch);
      kch[c] = ch * 8;
    }
  }
  __device__ __forceinline__ void load(const GemmArgs &, rsrc_t rs, int k0, int kend) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {                 // kend is a multiple of 8 here
      const int vo = k0 + kch[c] >= kend ? OOB : voff[c];
      raw[c][0] = ld_b128(rs, vo, k0 * 4);
      raw[c][1] = ld_b128(rs, vo + 16, k0 * 4);
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      if (tid + 256 * c < ROWS * 8) {
        if (HL) {
          uint4 h, l;
          h.x = __builtin_amdgcn_perm(raw[c][0].y, raw[c][0].x, 0x05040100u);
          h.y = __builtin_amdgcn_perm(raw[c][0].w, raw[c][0].z, 0x05040100u);
          h.z = __builtin_amdgcn_perm(raw[c][1].y, raw[c][1].x, 0x05040100u);
          h.w = __builtin_amdgcn_perm(raw[c][1].w, raw[c][1].z, 0x05040100u);
          l.x = __builtin_amdgcn_perm(raw[c][0].y, raw[c][0].x, 0x07060302u);
          l.y = __builtin_amdgcn_perm(raw[c][0].w, raw[c][0].z, 0x07060302u);
          l.z = __builtin_amdgcn_perm(raw[c][1].y, raw[c][1].x, 0x07060302u);
          l.w = __builtin_amdgcn_perm(raw[c][1].w, raw[c][1].z, 0x07060302u);
          *(uint4 *)(tile + loff[c]) = h;
          *(uint4 *)(tile + ROWS * 128 + loff[c]) = l;
        } else {
#pragma unroll
          for (int pl = 0; pl < 3; ++pl) {
            uint4 d;
            d.x = pack2(bf16_piece(__uint_as_float(raw[c][0].x), pl), bf16_piece(__uint_as_float(raw[c][0].y), pl));
            d.y = pack2(bf16_piece(__uint_as_float(raw[c][0].z), pl), bf16_piece(__uint_as_float(raw[c][0].w), pl));
            d.z = pack2(bf16_piece(__uint_as_float(raw[c][1].x), pl), bf16_piece(__uint_as_float(raw[c][1].y), pl));
            d.w = pack2(bf16_piece(__uint_as_float(raw[c][1].z), pl), bf16_piece(__uint_as_float(raw[c][1].w), pl));
            *(uint4 *)(tile + pl * ROWS * 128 + loff[c]) = d;
          }
        }
      }
    }
  }
};
template <int ROWS> struct LoaderP<P_HL, ROWS> : LoaderPWord<ROWS, true> {};
template <int ROWS> struct LoaderP<P_F32S, ROWS> : LoaderPWord<ROWS, false> {};

// P[m][i] bytes, contraction index m slowest.  One unit = 8 consecutive m x 8 consecutive i:
// eight 8-byte loads, one per row (a wavefront's loads of one row cover 256 consecutive bytes),
// transposed in registers into eight 16-byte LDS writes.
template <int ROWS> struct LoaderP<P_T_U8, ROWS> {
  static constexpr int PLANES = 1;
  static constexpr int UNITS = ROWS;                      // (ROWS/8) column groups x 8 m groups
  static constexpr int UP = (UNITS + 255) / 256;
  int voff[UP], loff[UP][8], mrow[UP];
  u32x2 raw[UP][8];
  // Rows are 4-byte aligned and the number of valid columns is a multiple of 4 (the host pads
  // the raster otherwise): no branches.  A unit that straddles the last valid column reads
  // what follows it in memory; those bytes only reach rows of the product that are not stored.
  __device__ __forceinline__ void setup(const GemmArgs &a, int row0, int tid) {
#pragma unroll
    for (int c = 0; c < UP; ++c) {
      const int u = tid + 256 * c;
      const int ig = u % (ROWS / 8), mg = u / (ROWS / 8);
      const int i = row0 + 8 * ig;
      voff[c] = (u < UNITS && i < a.p_ivalid) ? 8 * mg * a.ldp + i : OOB;
      mrow[c] = 8 * mg;
#pragma unroll
      for (int e = 0; e < 8; ++e) loff[c][e] = tile_off((8 * ig + e) & (ROWS - 1), mg & 7);
    }
  }
  __device__ __forceinline__ void load(const GemmArgs &a, rsrc_t rs, int k0, int kend) {
#pragma unroll
    for (int c = 0; c < UP; ++c) {
#pragma unroll
      for (int r = 0; r < 8; ++r)
        raw[c][r] = ld_b64(rs, k0 + mrow[c] + r >= kend ? OOB : voff[c], (k0 + r) * a.ldp);
    }
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < UP; ++c) {
      if (tid + 256 * c < UNITS) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          // byte e%4 of word e/4: of row 2h -> bits 0..7, of row 2h+1 -> bits 16..23
          const uint32_t sel = 0x0C000C00u | ((4u + (e & 3)) << 16) | (uint32_t)(e & 3);
          const int w = e >> 2;
          uint4 d;
          d.x = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][1][w], raw[c][0][w], sel));
          d.y = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][3][w], raw[c][2][w], sel));
          d.z = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][5][w], raw[c][4][w], sel));
          d.w = spikes2_to_bf16(__builtin_amdgcn_perm(raw[c][7][w], raw[c][6][w], sel));
          *(uint4 *)(tile + loff[c][e]) = d;
        }
      }
    }
  }
};

// P packed along time: bytes [ceil(T/8) * B][i], bit 7 - r of byte (tp, b, i) = the spike of channel
// i, sample b at step 8 tp + r.  Contraction in packed order: tile q covers packed rows 8q .. 8q+7
// (one tp, eight consecutive samples: B is a multiple of 8), k = 8 mg + r for sample mg of the
// eight and step r of the byte.  One unit = one sample x 8 consecutive i: a single 8-byte load,
// each byte expanded to the eight bfloat16 of one 16-byte chunk.  Bits of steps beyond T may hold
// anything: the rows of Q they meet read as zero.
template <int ROWS> struct LoaderP<P_T_BITS, ROWS> {
  static constexpr int PLANES = 1;
  static constexpr int UNITS = ROWS;                      // (ROWS/8) channel groups x 8 samples
  static constexpr int UP = (UNITS + 255) / 256;
  int voff[UP], loff[UP][8];
  u32x2 raw[UP];
  __device__ __forceinline__ void setup(const GemmArgs &a, int row0, int tid) {
#pragma unroll
    for (int c = 0; c < UP; ++c) {
      const int u = tid + 256 * c;
      const int ig = u % (ROWS / 8), mg = u / (ROWS / 8);
      const int i = row0 + 8 * ig;
      voff[c] = (u < UNITS && i < a.p_ivalid) ? mg * a.ldp + i : OOB;
#pragma unroll
      for (int e = 0; e < 8; ++e) loff[c][e] = tile_off((8 * ig + e) & (ROWS - 1), mg & 7);
    }
  }
  __device__ __forceinline__ void load(const GemmArgs &a, rsrc_t rs, int k0, int kend) {
#pragma unroll
    for (int c = 0; c < UP; ++c) raw[c] = ld_b64(rs, k0 >= kend ? OOB : voff[c], (k0 >> 3) * a.ldp);
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < UP; ++c) {
      if (tid + 256 * c < UNITS) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          // z holds the byte at bits 0..7 and again at bits 17..24: shifted right by 7 - 2j, bit 0 is
          // step 2j and bit 16 is step 2j + 1
          const uint32_t v = (raw[c][e >> 2] >> (8 * (e & 3))) & 0xFFu;
          const uint32_t z = v | (v << 17);
          uint4 d;
          d.x = ((z >> 7) & 0x00010001u) * 0x3F80u;
          d.y = ((z >> 5) & 0x00010001u) * 0x3F80u;
          d.z = ((z >> 3) & 0x00010001u) * 0x3F80u;
          d.w = ((z >> 1) & 0x00010001u) * 0x3F80u;
          *(uint4 *)(tile + loff[c][e]) = d;
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
  int voff[CH], loff[CH];
  u32x4 raw[NPL][CH];
  __device__ __forceinline__ void setup(const GemmArgs &a, int col0, int tid) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int cid = tid + 256 * c;
      const int r = cid >> 3, ch = cid & 7;
      voff[c] = cid < ROWS * 8 ? ((col0 + r) * a.ldq + ch * 8) * 2 : OOB;
      loff[c] = tile_off(r & (ROWS - 1), ch);
    }
  }
  __device__ __forceinline__ void load(const GemmArgs &a, rsrc_t rs, int k0, int kend) {
    const bool past = k0 >= kend;                  // uniform: a padding tile of the ring
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
      for (int c = 0; c < CH; ++c)
        raw[pl][c] = ld_b128(rs, past ? OOB : voff[c], (k0 + pl * (int)a.q_plane_stride) * 2);
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
      for (int c = 0; c < CH; ++c)
        if (tid + 256 * c < ROWS * 8) *(u32x4 *)(tile + pl * ROWS * 128 + loff[c]) = raw[pl][c];
  }
};

// Q[m][j] dwords, contraction index m slowest, ld a multiple of 8 with zero padding: HL words
// (two planes) or fp32 (three planes, split here).  One unit = 8 consecutive m x 4
// consecutive j: eight 16-byte loads, transposed into four 16-byte LDS writes per plane.
// PK: the contraction runs in the packed order of LoaderP<P_T_BITS>: tile q = k0 / 64 is packed row
// tp = q / (B/8) and samples 8 (q % (B/8)) .. +7; element 8 mg + r of the tile is row
// (8 tp + r) B + 8 (q % (B/8)) + mg of Q, and rows of steps beyond T read as zero.
template <int ROWS, bool HL, bool PK = false> struct LoaderQTWord {
  static constexpr int PLANES = HL ? 2 : 3;
  static constexpr int UNITS = ROWS * 2;
  static constexpr int UQ = (UNITS + 255) / 256;
  int voff[UQ], loff[UQ][4], mrow[UQ];
  u32x4 raw[UQ][8];
  __device__ __forceinline__ void setup(const GemmArgs &a, int col0, int tid) {
#pragma unroll
    for (int c = 0; c < UQ; ++c) {
      const int u = tid + 256 * c;
      const int jg = u % (ROWS / 4), mg = u / (ROWS / 4);
      const int j = col0 + 4 * jg;
      voff[c] = (u < UNITS && j < a.ldq) ? ((PK ? mg : 8 * mg) * a.ldq + j) * 4 : OOB;
      mrow[c] = 8 * mg;
#pragma unroll
      for (int e = 0; e < 4; ++e) loff[c][e] = tile_off((4 * jg + e) & (ROWS - 1), mg & 7);
    }
  }
  __device__ __forceinline__ void load(const GemmArgs &a, rsrc_t rs, int k0, int kend) {
    if (PK) {
      const int groups = a.pk_B >> 3, q = k0 >> 6;
      const int tp = q / groups, bg = q - tp * groups;
      const int row0 = 8 * tp * a.pk_B + 8 * bg;
#pragma unroll
      for (int c = 0; c < UQ; ++c)
#pragma unroll
        for (int r = 0; r < 8; ++r)
          raw[c][r] = ld_b128(rs, k0 >= kend || 8 * tp + r >= a.pk_T ? OOB : voff[c], (row0 + r * a.pk_B) * a.ldq * 4);
      return;
    }
#pragma unroll
    for (int c = 0; c < UQ; ++c)
#pragma unroll
      for (int r = 0; r < 8; ++r)
        raw[c][r] = ld_b128(rs, k0 + mrow[c] + r >= kend ? OOB : voff[c], (k0 + r) * a.ldq * 4);
  }
  __device__ __forceinline__ void store(char *tile, int tid) {
#pragma unroll
    for (int c = 0; c < UQ; ++c) {
      if (tid + 256 * c < UNITS) {
#pragma unroll
        for (int pl = 0; pl < PLANES; ++pl)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            uint4 d;
            if (HL) {
              const uint32_t sel = pl == 0 ? 0x05040100u : 0x07060302u;
              d.x = __builtin_amdgcn_perm(raw[c][1][e], raw[c][0][e], sel);
              d.y = __builtin_amdgcn_perm(raw[c][3][e], raw[c][2][e], sel);
              d.z = __builtin_amdgcn_perm(raw[c][5][e], raw[c][4][e], sel);
              d.w = __builtin_amdgcn_perm(raw[c][7][e], raw[c][6][e], sel);
            } else {
#define SNN_PC(r_) bf16_piece(__uint_as_float(raw[c][r_][e]), pl)
              d.x = pack2(SNN_PC(0), SNN_PC(1)); d.y = pack2(SNN_PC(2), SNN_PC(3));
              d.z = pack2(SNN_PC(4), SNN_PC(5)); d.w = pack2(SNN_PC(6), SNN_PC(7));
#undef SNN_PC
            }
            *(uint4 *)(tile + pl * ROWS * 128 + loff[c][e]) = d;
          }
      }
    }
  }
};
template <int ROWS, int NPL> struct LoaderQ<Q_T_HL, ROWS, NPL> : LoaderQTWord<ROWS, true> {
  static_assert(NPL == 2, "hi and lo");
};
template <int ROWS, int NPL> struct LoaderQ<Q_T_F32S, ROWS, NPL> : LoaderQTWord<ROWS, false> {
  static_assert(NPL == 3, "hi, mid and lo");
};
template <int ROWS, int NPL> struct LoaderQ<Q_T_HL_PK, ROWS, NPL> : LoaderQTWord<ROWS, true, true> {
  static_assert(NPL == 2, "hi and lo");
};
template <int ROWS, int NPL> struct LoaderQ<Q_T_F32S_PK, ROWS, NPL> : LoaderQTWord<ROWS, false, true> {
  static_assert(NPL == 3, "hi, mid and lo");
};

// ------------------------------------------------------------------ the kernel
// 256 threads = WM x WN wavefronts, each owning TM x TN MFMA tiles of 32x32.  One LDS stage.
// D register sets form a ring: the global loads of the next D tiles are always in flight, so
// that a workgroup alone keeps enough bytes outstanding to cover HBM/L2 latency even when
// few workgroups fit a compute unit.
// Bytes of the one LDS stage: every plane of both operand tiles.
template <int PM, int QM, int WM, int WN, int TM, int TN, int NQP>
constexpr int gemm_lds_bytes() {
  return LoaderP<PM, WM * TM * 32>::PLANES * WM * TM * 32 * 128 + NQP * WN * TN * 32 * 128;
}

template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP, int D>
__device__ __forceinline__ void gemm_body(const GemmArgs &a, const int block, char *lds) {
  static_assert(WM * WN == 4, "four wavefronts per workgroup");
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  typedef LoaderP<PM, BM> LP;
  typedef LoaderQ<QM, BN, NQP> LQ;
  constexpr int NPP = LP::PLANES;
  constexpr int NMAX = NPP > NQP ? NPP : NQP;
  constexpr int PT = BM * 128, QT = BN * 128;       // bytes of one plane of a tile
  constexpr int DR = D;
  static_assert(NPP * PT + NQP * QT <= 81920, "one stage, at least two workgroups per compute unit");

  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Without
  // contraction splits an XCD gets a contiguous run of tiles (column tiles fastest), so tiles
  // sharing a row slab of P share an L2.  With splits, XCD x takes the splits x, x+8, .. of
  // every tile: the tiles of one split read the same rows of both operands.
  const int ntiles = a.tiles_m * a.tiles_n;
  const int xcd = block & 7, slot = block >> 3;
  int tile, split;
  if (a.splits == 1) {
    tile = xcd * ((ntiles + 7) >> 3) + slot;
    split = 0;
  } else {
    tile = slot % ntiles;
    split = (slot / ntiles) * 8 + xcd;
  }
  if (tile >= ntiles || split >= a.splits) return;
  const int row0 = (tile / a.tiles_n) * BM;
  const int col0 = (tile % a.tiles_n) * BN;
  const int kbeg = split * a.kc_per_split;
  const int kend = min(a.kc, kbeg + a.kc_per_split);
  const int nk = kend > kbeg ? (kend - kbeg + 63) >> 6 : 0;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const rsrc_t rp = make_rsrc(a.P, a.p_bytes), rq = make_rsrc(a.Q, a.q_bytes);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  LP lp[DR];
  LQ lq[DR];
#pragma unroll
  for (int d = 0; d < DR; ++d) {
    lp[d].setup(a, row0, tid);
    lq[d].setup(a, col0, tid);
    lp[d].load(a, rp, kbeg + d * 64, kend);        // beyond kend the loads return zero
    lq[d].load(a, rq, kbeg + d * 64, kend);
  }

  // fragment addresses: row (lane & 31) of each 32-row block, chunk (lane >> 5) of step 0
  int fa[TM], fb[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) fa[i] = (wm * TM + i) * 32 + (lane & 31);
#pragma unroll
  for (int j = 0; j < TN; ++j) fb[j] = (wn * TN + j) * 32 + (lane & 31);

  // the products of one 64-wide contraction tile held in the stage at `st`
  auto multiply = [&](const char *st) {
    const char *sq = st + NPP * PT;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[NPP][TM], bq[NQP][TN];
      const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
      for (int p = 0; p < NPP; ++p)
#pragma unroll
        for (int i = 0; i < TM; ++i) af[p][i] = *(const bf16x8 *)(st + p * PT + tile_off(fa[i], chunk));
#pragma unroll
      for (int q = 0; q < NQP; ++q)
#pragma unroll
        for (int j = 0; j < TN; ++j) bq[q][j] = *(const bf16x8 *)(sq + q * QT + tile_off(fb[j], chunk));
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
  };

  {
    // One LDS stage.  The loop body is free of branches: the ring is run for a multiple of D
    // tiles and the tiles beyond the range load zeros.  (A load issued under a condition
    // would make every later wait conservative and serialise the ring.)
    const int nk_ring = (nk + DR - 1) / DR * DR;
    for (int kt0 = 0; kt0 < nk_ring; kt0 += DR) {
#pragma unroll
      for (int d = 0; d < DR; ++d) {
        lp[d].store(lds, tid);
        lq[d].store(lds + NPP * PT, tid);
        lp[d].load(a, rp, kbeg + (kt0 + d + DR) * 64, kend);
        lq[d].load(a, rq, kbeg + (kt0 + d + DR) * 64, kend);
        lds_barrier();
        multiply(lds);
        lds_barrier();                               // every wavefront is done with the stage
      }
    }
  }

  // Accumulator layout of the 32x32 MFMA: lane holds column (lane & 31); register r holds
  // row 8*(r/4) + 4*(lane/32) + (r%4).
  float *C = a.C + (size_t)split * a.c_split_stride;
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
          if (a.nt_store) __builtin_nontemporal_store(acc[i][j][r], &C[o]);
          else C[o] = acc[i][j][r];
        }
      }
    }
}

template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP, int D>
__global__ __launch_bounds__(256, 2) void gemm_kernel(const GemmArgs a) {
  __shared__ __attribute__((aligned(16))) char lds[gemm_lds_bytes<PM, QM, WM, WN, TM, TN, NQP>()];
  gemm_body<PM, QM, EPI, WM, WN, TM, TN, NQP, D>(a, blockIdx.x, lds);
}

// Several independent products of one kind in a single launch: a small product cannot fill
// the chip by itself, and every launch boundary costs a drain and a refill.  The workgroup
// ranges of the jobs start at multiples of 8, so that (id & 7) is still the XCD.
#define SNN_GEMM_MAX_JOBS 8
struct GemmJobs {
  int njobs;
  int first_block[SNN_GEMM_MAX_JOBS + 1];
  GemmArgs job[SNN_GEMM_MAX_JOBS];
};

template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP, int D>
__global__ __launch_bounds__(256, 2) void gemm_jobs_kernel(const GemmJobs jobs) {
  __shared__ __attribute__((aligned(16))) char lds[gemm_lds_bytes<PM, QM, WM, WN, TM, TN, NQP>()];
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first_block[j + 1]) ++j;
  if constexpr (PM == P_T_U8) {
    // a weight-gradient job on the raster packed along time: same tiles and stage, other loaders
    if (jobs.job[j].packed) {
      gemm_body<P_T_BITS, QM == Q_T_HL ? Q_T_HL_PK : Q_T_F32S_PK, EPI, WM, WN, TM, TN, NQP, D>(
          jobs.job[j], blockIdx.x - jobs.first_block[j], lds);
      return;
    }
  }
  gemm_body<PM, QM, EPI, WM, WN, TM, TN, NQP, D>(jobs.job[j], blockIdx.x - jobs.first_block[j], lds);
}

// Fills in the tile counts; returns the number of workgroups.
template <int WM, int WN, int TM, int TN>
static int gemm_prepare(GemmArgs &a, int splits) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  a.tiles_m = (a.rows + BM - 1) / BM;
  a.tiles_n = (a.cols + BN - 1) / BN;
  const int ntiles = a.tiles_m * a.tiles_n;
  a.splits = splits;
  return splits == 1 ? (ntiles + 7) / 8 * 8 : 8 * ntiles * ((splits + 7) / 8);
}

template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP, int D>
static hipError_t gemm_launch(GemmArgs a, int splits, hipStream_t st) {
  dim3 grid(gemm_prepare<WM, WN, TM, TN>(a, splits), 1, 1);
  hipLaunchKernelGGL((gemm_kernel<PM, QM, EPI, WM, WN, TM, TN, NQP, D>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

// Adds a job (its workgroup range) to a list launched later by gemm_jobs_launch.
template <int WM, int WN, int TM, int TN>
static void gemm_jobs_add(GemmJobs &jobs, GemmArgs a, int splits) {
  const int j = jobs.njobs++;
  const int blocks = gemm_prepare<WM, WN, TM, TN>(a, splits);
  jobs.job[j] = a;
  jobs.first_block[j + 1] = jobs.first_block[j] + blocks;
}

template <int PM, int QM, int EPI, int WM, int WN, int TM, int TN, int NQP, int D>
static hipError_t gemm_jobs_launch(const GemmJobs &jobs, hipStream_t st) {
  if (jobs.njobs == 0) return hipSuccess;
  dim3 grid(jobs.first_block[jobs.njobs], 1, 1);
  hipLaunchKernelGGL((gemm_jobs_kernel<PM, QM, EPI, WM, WN, TM, TN, NQP, D>), grid, dim3(256), 0, st, jobs);
  return hipGetLastError();
}

}  // namespace snn
