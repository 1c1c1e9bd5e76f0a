// Reverse pass of a whole feed-forward LIF layer below a narrow layer in one launch: the
// spike gradients dS = dX W^T from the current gradients dX of the layer above (at most 128
// columns: the readout or a narrow spiking layer), the surrogate, the reverse scan
// g_t -> dI_t (Eq. 1-2 differentiated; see lif_reverse_kernel), dI stored as hi/lo words.
//
// lif_reverse_top_kernel does the same with one wavefront per 64 chains, each lane walking
// its chain through global memory: per step a load, a store and a share of the dX fetches,
// which is what bounds it (a wavefront issues a memory instruction about every 60 cycles).
// Here a workgroup owns one sample and BN = 64 neurons (128 also builds; measured slower: one
// workgroup per compute unit, nothing overlaps its phases), and per block of 64 steps, last
// block first:
//   1. V (64 x BN) and dX (64 x ldc words) arrive through 16-byte loads issued one block
//      ahead (they land during the previous block's scan) and go to LDS;
//   2. dS: 32x32x16 bfloat16 MFMAs, the rounded weights of the wavefront's BN/2 neurons resident
//      in registers, the hi and lo halves of dX as the second operand, lo first; a wavefront
//      holds 32 steps x BN/2 neurons of the result;
//   3. still in the MFMA layout, every lane turns its elements into the two coefficients of
//      the step: with s = surr(V - theta), g' = beta g + s (dS - theta g) = c1 g + c2,
//      c1 = beta - s theta, c2 = s dS.  The surrogate (a division or an exponential) is
//      computed here by all four wavefronts, not inside the sequential scan;
//   4. scan: BN/64 wavefronts, one neuron per lane, 64 steps of one fused multiply-add each on
//      LDS (coefficients read 8 steps ahead, g written back in place of c2);
//   5. store: all wavefronts pack g into hi/lo words and write whole rows, 16 bytes per lane.
// g (and the decay gradient's partial sum) stay in the scanning lanes' registers from block
// to block.  Rows past T read as zero: c2 = 0 there and g, zero at the start, stays zero.
//
// WIDE: the layer above has more than 128 columns, so its weights no longer fit the registers and
// its current gradients no longer fit an LDS tile.  Step 2 then runs on the streamed pipeline of
// the forward products (WordTile below): both operands travel from memory straight into LDS in
// stages of 32 columns, the hi/lo words of dX are split into their two bfloat16 planes after the
// fragment read, and dS still never reaches memory.  The workgroup then owns 128 neurons.
#pragma once
#include "scan.hpp"
#include "gemm_stream.hpp"
#include <type_traits>

namespace snn {

// Streamed product for the reverse layer: acc^T (TN x 32 neurons by 32 steps per wavefront) =
// Q (rounded weights, rows = neurons n, bfloat16 [n][k]) times P^T (hi/lo words [row = step][k]),
// k = the columns of the layer above, for a tile of 64 steps x 64 TN neurons on 2 x 2 wavefronts.
// The pipeline is an earlier form of SpikeTile's (four stages of 32 k, one barrier per stage between
// a stage's two MFMA steps, loads issued three
// stages ahead as asm so that the compiler does not wait for them); what differs is the P
// operand: 128 bytes per row and stage, in eight 16-byte units; unit u of row r sits at slot
// u ^ (r % 8) (the permutation is applied on the global side of the direct-to-LDS loads) so
// that the fragment reads of 32 consecutive rows spread over all banks; a lane reads the eight
// words of its step and MFMA step, splits them into a hi and a lo fragment, and both meet the
// same Q fragment (lo first).
template <int TN, int NS>
struct WordTile {
  static constexpr int BM = 64, BN = 64 * TN;
  static constexpr int PT = BM * 128, QT = BN * 64, ST = PT + QT;
  static constexpr int PI = PT / 4096, QI = QT / 4096, NL = PI + QI;   // load instructions per wavefront and stage
  static_assert(NS >= 4, "the waits assume at least four stages");
  typedef u32x4 frag_t;

  static __device__ __forceinline__ int p_row(int wave, int lane, int q) { return 8 * (wave + 4 * q) + (lane >> 3); }
  static __device__ __forceinline__ int p_unit(int row, int lane) { return (lane & 7) ^ (row & 7); }
  static __device__ __forceinline__ int q_row(int wave, int lane, int q) { return 16 * (wave + 4 * q) + (lane >> 2); }
  static __device__ __forceinline__ int q_chunk(int row, int lane) { return (lane & 3) ^ ((row >> 2) & 3); }

  // pv: per-lane byte offsets of the wavefront's P loads (row start + 16 x unit, or OOB);
  // qv: of its Q loads.  nk: stages.  On return every load has landed and every wavefront is
  // past its last fragment read.
  static __device__ __forceinline__ void run(char *lds, const u32x4 rp, const u32x4 rq, const int (&pv)[PI],
                                             const int (&qv)[QI], const int nk, const int wave, const int lane,
                                             f32x16 (&acc)[TN]) {
    const int wm = wave >> 1, wn = wave & 1, h = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_ptr_t)lds;
    auto issue = [&](int kt_any, int buf) {
      const int kt = __builtin_amdgcn_readfirstlane(kt_any);
      u32x4 p = rp, qr = rq;
      if (kt >= nk) p.z = qr.z = 0;                  // beyond the contraction: same instruction count, nothing fetched
      const unsigned dst = __builtin_amdgcn_readfirstlane(lds0 + buf * ST + 1024 * wave);
#pragma unroll
      for (int q = 0; q < PI; ++q) load_to_lds_b128(p, dst + 4096 * q, pv[q], kt * 128);
#pragma unroll
      for (int q = 0; q < QI; ++q) load_to_lds_b128(qr, dst + PT + 4096 * q, qv[q], kt * 64);
    };
    // fragment addresses: P row ra, units 4 st + 2 h and + 1 of MFMA step st; Q row rb, chunk 2 st + h
    int fa[2][2], fb[2];
    {
      const int ra = 32 * wm + (lane & 31), rb = wn * TN * 32 + (lane & 31);
#pragma unroll
      for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int e = 0; e < 2; ++e) fa[st][e] = ra * 128 + (((4 * st + 2 * h + e) ^ (ra & 7)) << 4);
        fb[st] = PT + rb * 64 + (((2 * st + h) ^ ((rb >> 2) & 3)) << 4);    // k = 16 st + 8 h .. + 7, as on the P side
      }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    auto read_first = [&](int buf, frag_t (&pa)[2][2], frag_t (&qb)[TN]) {   // P words of a stage, Q of its step 0
      const char *st = lds + buf * ST;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int e = 0; e < 2; ++e) pa[s2][e] = *(const frag_t *)(st + fa[s2][e]);
#pragma unroll
      for (int j = 0; j < TN; ++j) qb[j] = *(const frag_t *)(st + fb[0] + j * 2048);
    };
    auto products = [&](const frag_t (&pa)[2][2], const frag_t (&qb)[TN], int st) {
      const frag_t j0 = pa[st][0], j1 = pa[st][1];
      u32x4 hh, ll;
      hh.x = __builtin_amdgcn_perm(j0.y, j0.x, 0x05040100u); ll.x = __builtin_amdgcn_perm(j0.y, j0.x, 0x07060302u);
      hh.y = __builtin_amdgcn_perm(j0.w, j0.z, 0x05040100u); ll.y = __builtin_amdgcn_perm(j0.w, j0.z, 0x07060302u);
      hh.z = __builtin_amdgcn_perm(j1.y, j1.x, 0x05040100u); ll.z = __builtin_amdgcn_perm(j1.y, j1.x, 0x07060302u);
      hh.w = __builtin_amdgcn_perm(j1.w, j1.z, 0x05040100u); ll.w = __builtin_amdgcn_perm(j1.w, j1.z, 0x07060302u);
      const bf16x8 hi = __builtin_bit_cast(bf16x8, hh), lo = __builtin_bit_cast(bf16x8, ll);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, qb[j]), lo, acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, qb[j]), hi, acc[j], 0, 0, 0);
    };
    auto stage = [&](int u, int kt, frag_t (&pa)[2][2], frag_t (&qb)[TN], frag_t (&pa_next)[2][2], frag_t (&qb_next)[TN]) {
      frag_t q1[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) q1[j] = *(const frag_t *)(lds + u * ST + fb[1] + j * 2048);
      products(pa, qb, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(acc[j]));
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * NL) : "memory");   // younger stages may still be in flight
      lds_barrier();
      issue(kt + NS - 1, (u + NS - 1) % NS);
      read_first((u + 1) % NS, pa_next, qb_next);
      products(pa, q1, 1);
    };
#pragma unroll
    for (int t = 0; t < NS - 1; ++t) issue(t, t);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NL) : "memory");
    lds_barrier();
    frag_t pa0[2][2], qb0[TN], pa1[2][2], qb1[TN];
    read_first(0, pa0, qb0);
    constexpr int UN = NS % 2 ? 2 * NS : NS;
    for (int kt = 0; kt < nk; kt += UN) {
      bool done = false;
      static_for<UN>([&](auto U) {
        constexpr int u = decltype(U)::value;
        if (!done) {
          if constexpr (u % 2 == 0) stage(u % NS, kt + u, pa0, qb0, pa1, qb1);
          else stage(u % NS, kt + u, pa1, qb1, pa0, qb0);
          if (kt + u + 1 >= nk) done = true;
        }
      });
      if (done) break;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
  }
};

struct LayerReverseArgs {
  const uint32_t *dX;      // current gradients of the layer above [T*B][ldc], hi/lo words
  int ldc;                 // its padded columns (multiple of 8, at most 128)
  const uint16_t *Wq;      // rounded W[n][c] bfloat16, row n = neuron of this layer, zero beyond the valid columns
  int ldq;
  unsigned wq_bytes;
  const float *V;          // [T*B][ld]
  uint32_t *dI;            // [T*B][ld] hi/lo words
  const float *beta_v;     // [ld]
  float theta, slope;
  float *db_part;          // [B][ld] per-sample parts of the decay gradient, or NULL
  int T, B, ld;            // ld: a multiple of the workgroup's neurons
  int nt_store;            // dI streams past the caches
};

template <int KS, int SURR, int BN, bool WIDE = false>
__global__ __launch_bounds__(256, BN == 64 ? 2 : 1) void lif_layer_reverse_kernel(const LayerReverseArgs a) {
  static_assert(BN == 64 || BN == 128, "neurons per workgroup");
  static_assert(!WIDE || (BN == 128 && KS == 1), "the streamed product takes 128 neurons; KS has no meaning there");
  typedef WordTile<2, 4> Wide;
  constexpr int BM = 64;
  constexpr int NJ = BN / 64;                         // 32-neuron MFMA tiles per wavefront
  constexpr int NV = BN / 16;                         // 16-byte accesses per thread to a 64 x BN fp32 tile
  constexpr int LPR = BN / 4;                         // lanes per row in those accesses
  constexpr int CP = BN * 4 + 16;                     // bytes between time rows of the fp32 tiles
  constexpr int PITCH = CP / 4;
  constexpr int XP = KS * 128 + 16;                   // bytes between time rows of the dX tile (32 KS words)
  constexpr int TILE = BM * CP;
  constexpr int KK = 2 * KS;                          // 16-wide MFMA steps over the columns above
  static_assert(BM * XP <= 2 * TILE, "the dX tile shares the space of the coefficient tiles");
  static_assert(!WIDE || (4 * Wide::ST <= 2 * TILE && TILE % 1024 == 0), "the stages share the space of the coefficient tiles");
  __shared__ __attribute__((aligned(16))) char lds[3 * TILE];
  __shared__ __attribute__((aligned(16))) float betas[BN];
  char *const Vt = lds, *const C1 = lds + TILE, *const C2 = lds + 2 * TILE, *const Xt = C1;

  // Workgroup ids are dealt round-robin to the 8 XCDs: the parts of a sample take ids 8 apart.
  const int parts = a.ld / BN;
  const int part = (blockIdx.x >> 3) % parts;
  const int b = (blockIdx.x >> 3) / parts * 8 + (blockIdx.x & 7);
  if (b >= a.B) return;
  const int n0 = part * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, h = lane >> 5;
  const float theta = a.theta, slope = a.slope;
  const unsigned vbytes = (unsigned)a.T * a.B * a.ld * 4u;
  const rsrc_t rV = make_rsrc(a.V, vbytes), rdI = make_rsrc(a.dI, vbytes);
  const rsrc_t rX = make_rsrc(a.dX, (unsigned)a.T * a.B * a.ldc * 4u), rW = make_rsrc(a.Wq, a.wq_bytes);
  if (tid < BN) betas[tid] = a.beta_v[n0 + tid];

  // A block's global loads: V as 8 x 16 bytes per thread (row = 8 k + tid / 32), dX as KK x 16
  // bytes per thread over rows of 8 KS chunks (chunks beyond ldc read as zero).
  u32x4 xv[NV], xd[KK];
  auto fetch = [&](int t0) {                          // t0 < 0: nothing is read
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int t = t0 + (256 / LPR) * k + tid / LPR, col = (tid % LPR) * 4;
      xv[k] = ld_b128(rV, t0 >= 0 && t < a.T ? ((t * a.B + b) * a.ld + n0 + col) * 4 : OOB, 0);
    }
    if (!WIDE) {
#pragma unroll
      for (int k = 0; k < KK; ++k) {
        const int idx = k * 256 + tid, row = idx / (8 * KS), ch = idx % (8 * KS), t = t0 + row;
        xd[k] = ld_b128(rX, t0 >= 0 && t < a.T && ch * 4 + 3 < a.ldc ? ((t * a.B + b) * a.ldc + ch * 4) * 4 : OOB, 0);
      }
    }
  };
  auto fill = [&]() {
#pragma unroll
    for (int k = 0; k < NV; ++k) *(u32x4 *)(Vt + ((256 / LPR) * k + tid / LPR) * CP + (tid % LPR) * 16) = xv[k];
    if (!WIDE) {
#pragma unroll
      for (int k = 0; k < KK; ++k) {
        const int idx = k * 256 + tid, row = idx / (8 * KS), ch = idx % (8 * KS);
        *(u32x4 *)(Xt + row * XP + ch * 16) = xd[k];
      }
    }
  };

  int t0 = (a.T - 1) / BM * BM;
  fetch(t0);                                          // the first block's loads go out before anything else

  // First MFMA operand: W[n][c], lane -> neuron (lane & 31) of the 32-neuron tile, columns
  // 16 kk + 8 h .. +7.  Resident for the whole kernel.
  bf16x8 wf[NJ][KK];
  if (!WIDE) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const int n = n0 + 32 * NJ * wn + 32 * j + (lane & 31), c = 16 * kk + 8 * h;
        wf[j][kk] = __builtin_bit_cast(bf16x8, ld_b128(rW, c + 7 < a.ldq ? (n * a.ldq + c) * 2 : OOB, 0));
      }
  }
  // WIDE: global side of the streamed loads.  Q rows are this workgroup's neurons; P rows are the
  // block's steps (set per block).
  const u32x4 rpw = raw_rsrc(a.dX, (unsigned)a.T * a.B * a.ldc * 4u), rqw = raw_rsrc(a.Wq, a.wq_bytes);
  int qvw[Wide::QI];
#pragma unroll
  for (int q = 0; q < Wide::QI; ++q) {
    const int row = Wide::q_row(wave, lane, q);
    qvw[q] = ((n0 + row) * a.ldq + Wide::q_chunk(row, lane) * 8) * 2;
  }
  const int nkw = (a.ldc + 31) >> 5;

  float g = 0.f, db = 0.f;                            // state of neuron n0 + tid (wavefronts 0 and 1)

  for (int blk = 0; t0 >= 0; t0 -= BM, ++blk) {
    fill();
    __syncthreads();
    fetch(t0 - BM);

    // 2. dS^T tile: rows = neurons, columns = steps; the lane holds step 32 wm + (lane & 31)
    // and register r neuron 8 (r / 4) + 4 h + (r % 4) of its 32-neuron tile.
    f32x16 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    if constexpr (WIDE) {
      int pvw[Wide::PI];
#pragma unroll
      for (int q = 0; q < Wide::PI; ++q) {
        const int row = Wide::p_row(wave, lane, q), t = t0 + row;
        pvw[q] = t < a.T ? ((t * a.B + b) * a.ldc) * 4 + Wide::p_unit(row, lane) * 16 : OOB;
      }
      Wide::run(C1, rpw, rqw, pvw, qvw, nkw, wave, lane, acc);
    } else {
      bf16x8 hi[KK];
      const char *px = Xt + (32 * wm + (lane & 31)) * XP + 32 * h;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const u32x4 j0 = *(const u32x4 *)(px + 64 * kk), j1 = *(const u32x4 *)(px + 64 * kk + 16);
        u32x4 hh, ll;
        hh.x = __builtin_amdgcn_perm(j0.y, j0.x, 0x05040100u); ll.x = __builtin_amdgcn_perm(j0.y, j0.x, 0x07060302u);
        hh.y = __builtin_amdgcn_perm(j0.w, j0.z, 0x05040100u); ll.y = __builtin_amdgcn_perm(j0.w, j0.z, 0x07060302u);
        hh.z = __builtin_amdgcn_perm(j1.y, j1.x, 0x05040100u); ll.z = __builtin_amdgcn_perm(j1.y, j1.x, 0x07060302u);
        hh.w = __builtin_amdgcn_perm(j1.w, j1.z, 0x05040100u); ll.w = __builtin_amdgcn_perm(j1.w, j1.z, 0x07060302u);
        hi[kk] = __builtin_bit_cast(bf16x8, hh);
        const bf16x8 lo = __builtin_bit_cast(bf16x8, ll);
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j][kk], lo, acc[j], 0, 0, 0);
      }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j][kk], hi[kk], acc[j], 0, 0, 0);
    }
    __syncthreads();                                  // every wavefront has read the dX tile: C1 takes its place

    // 3. coefficients
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int t = 32 * wm + (lane & 31), n = 32 * NJ * wn + 32 * j + 8 * q + 4 * h;
        const f32x4 vv = *(const f32x4 *)(Vt + t * CP + n * 4);
        const f32x4 bb = *(const f32x4 *)(&betas[n]);
        f32x4 c1, c2;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float s = surr_rcp<SURR>(slope, vv[e] - theta);
          c1[e] = bb[e] - s * theta;
          c2[e] = s * acc[j][4 * q + e];
        }
        *(f32x4 *)(C1 + t * CP + n * 4) = c1;
        *(f32x4 *)(C2 + t * CP + n * 4) = c2;
      }
    __syncthreads();

    // 4. scan, steps t0 + 63 down to t0: dI_t = g, then g <- c1 g + c2 (and db += g V_t)
    if (wave < BN / 64) {
      const float *p1 = (const float *)(C1 + tid * 4), *pv = (const float *)(Vt + tid * 4);
      float *p2 = (float *)(C2 + tid * 4);
      auto scan = [&](auto DB) {
        constexpr bool with_db = decltype(DB)::value;
        constexpr int U = 8;
        float n1[U], n2[U], nv[U];
        auto read = [&](int s0) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            n1[u] = p1[(s0 + u) * PITCH];
            n2[u] = p2[(s0 + u) * PITCH];
            if (with_db) nv[u] = pv[(s0 + u) * PITCH];
          }
        };
        read(BM - U);
        for (int s0 = BM - U; s0 >= 0; s0 -= U) {
          float c1[U], c2[U], vv[U];
#pragma unroll
          for (int u = 0; u < U; ++u) { c1[u] = n1[u]; c2[u] = n2[u]; vv[u] = with_db ? nv[u] : 0.f; }
          if (s0 >= U) read(s0 - U);                  // the next 8 steps' coefficients, before these 8 are taken
#pragma unroll
          for (int u = 0; u < U; ++u) asm volatile("" : "+v"(c1[u]), "+v"(c2[u]));
#pragma unroll
          for (int u = U - 1; u >= 0; --u) {
            p2[(s0 + u) * PITCH] = g;
            if (with_db) db = __builtin_fmaf(g, vv[u], db);
            g = __builtin_fmaf(c1[u], g, c2[u]);
          }
        }
      };
      if (a.db_part) scan(std::true_type()); else scan(std::false_type());
    }
    __syncthreads();

    // 5. store: BN/4 lanes x 16 bytes per row
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int row = (256 / LPR) * k + tid / LPR, col = (tid % LPR) * 4, t = t0 + row;
      const f32x4 gq = *(const f32x4 *)(C2 + row * CP + col * 4);
      u32x4 w;
      w.x = pack_hl(gq[0]); w.y = pack_hl(gq[1]); w.z = pack_hl(gq[2]); w.w = pack_hl(gq[3]);
      const int vo = t < a.T ? ((t * a.B + b) * a.ld + n0 + col) * 4 : OOB;
      if (a.nt_store) __builtin_amdgcn_raw_buffer_store_b128(w, rdI, vo, 0, NT);
      else __builtin_amdgcn_raw_buffer_store_b128(w, rdI, vo, 0, 0);
    }
    // The next block's fill writes V and dX, which takes the place of C1 and, when its rows are
    // longer than a coefficient row, of part of C2, which this store phase is still reading.
    if (XP > CP) __syncthreads();
  }
  if (a.db_part && tid < BN) a.db_part[b * a.ld + n0 + tid] = db;
}

}  // namespace snn
