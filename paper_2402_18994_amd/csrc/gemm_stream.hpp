// The current product I = S W for large layers, gfx950: C[i][j] = sum_k P(i,k) * Q(j,k) with
// P the 0/1 spike bytes [row][k] and Q one bfloat16 plane of W^T [j][k] (rounded weights).
//
// The general product kernel stages operand tiles through registers: wait for the global
// loads, convert, write to LDS, issue the next loads, barrier, multiply, barrier.  Measured
// on the part, every phase is bound by what one wavefront can issue (a 16-byte LDS write
// about every 36 cycles, a buffer load about every 60), and the phases of a workgroup do not
// overlap.  This kernel removes the staging phase instead of hiding it:
//
//   * both operand tiles travel from memory straight into LDS (buffer_load ... lds, 16 bytes
//     per lane): no staging registers, no LDS write instructions, no conversion before the
//     barrier.  A wavefront's 64 lanes fill 1 KiB of consecutive LDS, so the bank swizzle is
//     applied on the global side: each lane fetches the 16-byte unit that belongs at its slot;
//   * the spikes stay bytes in LDS (half the LDS traffic of the P operand) and become
//     bfloat16 in registers, after the fragment read, between the MFMAs;
//   * four LDS stages of 32 contraction elements and one barrier per stage: the loads of
//     stage t+3 are issued during stage t and have almost three stages to land (the P operand
//     comes from HBM on first touch; two stages of 64 left a third of a microsecond of wait
//     per tile);
//   * fragments are read one MFMA step ahead of their use, across the stage boundary too:
//     the barrier sits between the two steps of a stage.
//
// Contraction order inside a stage.  A lane holds 8 consecutive k per MFMA.  Reading a lane's
// P bytes 16 at a time (two steps' worth) fixes which k a step covers: step s of lane half
// h = lane/32 covers k = 16h + 8s .. +7, and the Q fragment of that step is read from the
// matching 16-byte chunk 2h + s of the row.
//
// Tails.  Rows of P beyond the product read as zero (lane offset beyond the buffer).  Along
// k nothing is masked on the P side: Q is zero-padded to a multiple of 64 along k, and
// whatever bytes P yields there are reduced to 0/1 before they meet those zeros.
#pragma once
#include "gemm.hpp"
#include <type_traits>

namespace snn {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// 16 bytes per lane from a buffer straight into LDS: lane L's bytes land at lds_addr + 16 L
// (lds_addr: byte address within LDS, the same for the whole wavefront); a lane whose offset
// is beyond the buffer writes zeros.  Written as asm on purpose.  The compiler would guard
// every later LDS read it cannot tell apart from such a load's target with a wait for the
// load, and at a loop head with a wait for all loads in flight, which undoes a prefetch
// distance of several stages.  This way the loads are invisible to it: the kernel waits
// explicitly (vmcnt) and orders with barriers.  The descriptor is the usual raw buffer
// resource (base, 0 stride, size, 0x00020000); M0 carries the LDS address and has no other
// use in a kernel that includes this.
__device__ __forceinline__ u32x4 raw_rsrc(const void *base, unsigned bytes) {
  const unsigned long long b = (unsigned long long)base;
  u32x4 r;
  r.x = (unsigned)b;
  r.y = (unsigned)(b >> 32) & 0xFFFFu;
  r.z = bytes;
  r.w = 0x00020000u;
  return r;
}
__device__ __forceinline__ void load_to_lds_b128(u32x4 rsrc, unsigned lds_addr, int voff, int soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}

template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>());
  }
}

// P operand packed along time (the storage format of Section 2.1.4: eight consecutive steps of one
// channel in a byte, first step in the most significant bit), for tiles whose 128 rows are
// consecutive time steps of one sample: the 16 packed rows of the block.
struct PackedRows {
  rsrc_t rsrc;         // the packed raster
  int base;            // byte offset of the block's first packed row for this sample
  int row_stride;      // bytes between packed rows of the sample (B x row length)
  int rows;            // packed rows that exist from there on (others read as zero)
  int kbytes;          // row length in bytes (= fan-in), at most 1024, a multiple of 4
};

// Geometry and main loop of one tile, shared by the kernels built on this pipeline.  `run`
// expects the per-lane global offsets of the wavefront's load instructions (pv: P, row-major
// bytes; qv: Q, bfloat16), takes the stages through `lds` (NS * ST bytes) and leaves the
// products in acc; on return every load has landed and every wavefront is past its last
// fragment read, so the caller may reuse the LDS.
template <int WM, int WN, int TM, int TN, int NS>
struct SpikeTile {
  static_assert(WM * WN == 4, "four wavefronts per workgroup");
  static constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  // (a tile of 64 rows still gives P a whole KiB per wavefront and stage: the rows beyond the tile
  // are loaded as rows outside the product, i.e. as zeros, and never read)
  static constexpr int PT = (BM < 128 ? 128 : BM) * 32, QT = BN * 64, ST = PT + QT;   // bytes: P part, Q part, stage (32 k)
  static constexpr int PI = PT / 4096, QI = BN / 64;                // load instructions per wavefront and stage
  static constexpr int NL = PI + QI;
  static_assert(BM % 64 == 0 && BN % 64 == 0, "whole KiB per wavefront");
  static_assert(NS >= 4, "the waits assume at least four stages");
  typedef u32x4 frag_t;
  // Packed P operand: the whole block of the sample (BM / 8 packed rows of up to 1024 bytes) sits
  // in LDS for all stages, ahead of the stages, which then hold Q alone.  A row pitch of 1088 bytes
  // puts the four packed rows a fragment read touches on different banks.
  static constexpr int PKP = 1088, PKB = ((BM / 8) * PKP + 1023) / 1024 * 1024;   // (the stages behind it start on a KiB)
  static constexpr int lds_bytes(bool pk) { return pk ? PKB + NS * QT : NS * ST; }

  // Global side of the loads.  P instruction q of a wavefront fills rows 32 (wave + 4 q) ..
  // +31 of the stage, 32 bytes each: lane -> row lane/2, slot lane%2, which holds the 16-byte
  // unit slot ^ ((row / 8) % 2).  Q instruction q fills rows 16 (wave + 4 q) .. +15, 64 bytes
  // each: lane -> row lane/4, slot lane%4, holding the 16-byte chunk slot ^ ((row / 4) % 4).
  // With these permutations the fragment reads (32 consecutive rows, one unit or chunk)
  // touch every bank equally.
  static __device__ __forceinline__ int p_row(int wave, int lane, int q) { return 32 * (wave + 4 * q) + (lane >> 1); }
  static __device__ __forceinline__ int p_unit(int row, int lane) { return (lane & 1) ^ ((row >> 3) & 1); }
  static __device__ __forceinline__ int q_row(int wave, int lane, int q) { return 16 * (wave + 4 * q) + (lane >> 2); }
  static __device__ __forceinline__ int q_chunk(int row, int lane) { return (lane & 3) ^ ((row >> 2) & 3); }

  // PK: P comes from `pk` (packed along time; BM == 128 rows = time steps of one sample) instead
  // of rp / pv: a lane's 16 bytes of row r, columns 16 h .. +15 of a stage, are bit 7 - r % 8 of
  // the 16 packed bytes at packed row r / 8; no P loads per stage.
  template <bool PK = false>
  static __device__ __forceinline__ void run(char *lds, const u32x4 rp, const u32x4 rq, const int (&pv)[PI],
                                             const int (&qv)[QI], const int nk, const int wave, const int lane,
                                             f32x16 (&acc)[TM][TN], const PackedRows *pk = nullptr) {
    const int wm = wave / WN, wn = wave % WN;
    constexpr int STQ = PK ? QT : ST;               // bytes of a stage
    constexpr int QOFF = PK ? 0 : PT;               // where Q starts inside a stage
    constexpr int NLK = PK ? QI : NL;               // load instructions per wavefront and stage
    char *const stages = lds + (PK ? PKB : 0);
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_ptr_t)stages;
    constexpr int PKN = BM / 32;                    // 16-byte pieces of the packed block per thread
    u32x4 pkx[PKN];
    if (PK) {
      // the block's packed rows: BM / 8 rows x 64 pieces of 16 bytes, BM / 32 pieces per thread;
      // pieces beyond the last packed row or the row length read as zero
      const int tid = 64 * wave + lane;
#pragma unroll
      for (int j = 0; j < PKN; ++j) {
        const int piece = tid + 256 * j, r = piece >> 6, c = (piece & 63) * 16;
        pkx[j] = ld_b128(pk->rsrc, r < pk->rows && c < pk->kbytes ? r * pk->row_stride + c : OOB, pk->base);
      }
    }
    // Stage kt into buffer `buf`.  Beyond the contraction range the descriptors get size 0:
    // the instruction count (which the vmcnt waits rely on) stays the same, nothing is fetched.
    struct IssueRegs {                                  // scalar operands of one stage's loads
      u32x4 p, q;
      unsigned dst;
      int kt;
    };
    auto issue_prepare = [&](int kt_any, int buf) {
      IssueRegs r;
      r.kt = __builtin_amdgcn_readfirstlane(kt_any);          // uniform; keeps the offsets scalar
      r.p = rp; r.q = rq;
      if (r.kt >= nk) r.p.z = r.q.z = 0;
      r.dst = __builtin_amdgcn_readfirstlane(lds0 + buf * STQ + 1024 * wave);
      asm volatile("" : "+s"(r.p.z), "+s"(r.q.z), "+s"(r.dst), "+s"(r.kt));   // formed here, not next to the loads
      return r;
    };
    auto issue_load = [&](const IssueRegs &r, int n) {        // load instruction n of the stage (P first)
      if (n < NLK - QI) load_to_lds_b128(r.p, r.dst + 4096 * n, pv[n < PI ? n : 0], r.kt * 32);
      else load_to_lds_b128(r.q, r.dst + QOFF + 4096 * (n - (NLK - QI)), qv[n - (NLK - QI)], r.kt * 64);
    };
    auto issue = [&](int kt_any, int buf) {
      const IssueRegs r = issue_prepare(kt_any, buf);
#pragma unroll
      for (int n = 0; n < NLK; ++n) issue_load(r, n);
    };

    // LDS side of the fragment reads: lane half h reads P unit h (16 k, two MFMA steps' worth)
    // and, for step s, Q chunk 2h + s.  Rows 32 apart share the permutation.
    const int h = lane >> 5;
    int fa, fb[2];
    {
      const int ra = wm * TM * 32 + (lane & 31), rb = wn * TN * 32 + (lane & 31);
      fa = PK ? (ra >> 3) * PKP + 16 * h : ra * 32 + ((h ^ ((ra >> 3) & 1)) << 4);
#pragma unroll
      for (int st = 0; st < 2; ++st) fb[st] = QOFF + rb * 64 + (((2 * h + st) ^ ((rb >> 2) & 3)) << 4);
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Registers of one stage: its P bytes, spread (a spike is 0x40 in its byte), the Q fragments of
    // its MFMA step 0, and the P fragments of step 0.
    struct StageRegs {
      frag_t pa[TM], qb[TN];
      bf16x8 af[TM];
    };
    // Spike bytes to bfloat16 with two instructions per four spikes.  0x40 in the upper byte of a
    // bfloat16 is 2.0, so a spike byte becomes an operand by one shift of its dword (0/1 -> 0x00/0x40
    // in each byte; from the packed form: a rotation that brings the lane's bit to bit 6 of every
    // byte, and a mask) and one byte permutation per pair.  The products come out doubled, exactly
    // (a power of two), and are halved after the last stage.
    // (the lane's step is bit 7 - lane % 8 of a packed byte: a rotation to the right by that minus 6, mod 32)
    const unsigned pk_rot = (unsigned)(1 - (lane & 7)) & 31u;
    auto spread = [&](frag_t &w) {
#pragma unroll
      for (int d = 0; d < 4; ++d)
        w[d] = PK ? (__builtin_amdgcn_alignbit(w[d], w[d], pk_rot) & 0x40404040u) : (w[d] << 6);
    };
    auto convert = [&](uint32_t t0, uint32_t t1) {
      u32x4 d;
      d.x = __builtin_amdgcn_perm(0u, t0, 0x010C000Cu);
      d.y = __builtin_amdgcn_perm(0u, t0, 0x030C020Cu);
      d.z = __builtin_amdgcn_perm(0u, t1, 0x010C000Cu);
      d.w = __builtin_amdgcn_perm(0u, t1, 0x030C020Cu);
      return __builtin_bit_cast(bf16x8, d);
    };
    auto read_first = [&](int buf, int kt, StageRegs &r) {    // P bytes of stage kt (as stored), Q of its step 0
      const char *st = stages + buf * STQ;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        r.pa[i] = PK ? *(const frag_t *)(lds + fa + i * 4 * PKP + kt * 32) : *(const frag_t *)(st + fa + i * 1024);
#pragma unroll
      for (int j = 0; j < TN; ++j) r.qb[j] = *(const frag_t *)(st + fb[0] + j * 2048);
    };
    // One stage in buffer u.  On entry the stage's P bytes, its step-0 Q fragments and its converted
    // step-0 P fragments are in registers (or on their way).  The barrier sits between the two MFMA
    // steps: past it, every wavefront has left stage kt-1 (its buffer, u+NS-1, may be overwritten:
    // the loads of stage kt+NS-1 go there) and has seen its own loads of stage kt+1 land (so buffer
    // u+1 is complete and its first fragments can be read under the MFMAs of step 1).
    //
    // One wavefront per SIMD: nothing but this wavefront's own independent instructions fills the
    // 32 cycles an MFMA keeps the matrix unit.  The order is therefore fixed by hand (scheduling
    // barriers), one MFMA, then the few conversion instructions of a fragment needed later:
    // step 1's fragments under the MFMAs of step 0, the next stage's step-0 fragments under the last
    // MFMAs of step 1, the fragment reads and the load issue right behind the barrier under the
    // first ones.  Left to the scheduler, the conversions of a whole stage sit in front of its first
    // MFMA and the fragment reads of a stage at its top, each followed by its wait.
    auto pin = [&](bf16x8 &f) {                             // the fragment is formed here, not next to its use
      u32x4 x = __builtin_bit_cast(u32x4, f);
      asm volatile("" : "+v"(x));
      f = __builtin_bit_cast(bf16x8, x);
    };
    auto stage = [&](int u, int kt, StageRegs &cur, StageRegs &nxt) {
      constexpr int M = TM * TN;                        // MFMAs per step
      frag_t q1[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) q1[j] = *(const frag_t *)(stages + u * STQ + fb[1] + j * 2048);
      bf16x8 a1[TM];
      IssueRegs ir;
      __builtin_amdgcn_sched_barrier(0);
      static_for<M>([&](auto X) {
        constexpr int x = decltype(X)::value, i = x / TN, j = x % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cur.qb[j]), cur.af[i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (x < TM) {
          a1[x] = convert(cur.pa[x][2], cur.pa[x][3]);
          pin(a1[x]);
        }
        if constexpr (x == (TM < M - 1 ? TM : M - 1)) ir = issue_prepare(kt + NS - 1, (u + NS - 1) % NS);
        __builtin_amdgcn_sched_barrier(0);
      });
      // (ties the accumulators to this point: the MFMAs of step 0 are issued before the waits)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(acc[i][j]));
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * NLK) : "memory");   // younger stages may still be in flight
      lds_barrier();
      {
        const char *st = stages + ((u + 1) % NS) * STQ;
#pragma unroll
        for (int i = 0; i < TM; ++i)
          nxt.pa[i] = PK ? *(const frag_t *)(lds + fa + i * 4 * PKP + (kt + 1) * 32) : *(const frag_t *)(st + fa + i * 1024);
      }
      __builtin_amdgcn_sched_barrier(0);
      constexpr int L0 = M - TM >= 2 ? (NLK < 2 ? NLK : 2) : NLK;   // load instructions behind the first MFMA
      static_for<M>([&](auto X) {
        constexpr int x = decltype(X)::value, i = x / TN, j = x % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q1[j]), a1[i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (x == 0) {
#pragma unroll
          for (int n = 0; n < L0; ++n) issue_load(ir, n);
        }
        if constexpr (x == (L0 < NLK ? 1 : 0)) {
#pragma unroll
          for (int n = L0; n < NLK; ++n) issue_load(ir, n);
          const char *st = stages + ((u + 1) % NS) * STQ;
#pragma unroll
          for (int jj = 0; jj < TN; ++jj) nxt.qb[jj] = *(const frag_t *)(st + fb[0] + jj * 2048);
        }
        if constexpr (x >= M - TM) {
          constexpr int i2 = x - (M - TM);
          spread(nxt.pa[i2]);
          nxt.af[i2] = convert(nxt.pa[i2][0], nxt.pa[i2][1]);
          pin(nxt.af[i2]);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    };

#pragma unroll
    for (int t = 0; t < NS - 1; ++t) issue(t, t);
    if (PK) {
      // (the wait the compiler puts before these writes covers the stage loads issued above as
      // well: memory returns loads in order)
      const int tid = 64 * wave + lane;
#pragma unroll
      for (int j = 0; j < PKN; ++j) {
        const int piece = tid + 256 * j;
        *(u32x4 *)(lds + (piece >> 6) * PKP + (piece & 63) * 16) = pkx[j];
      }
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NLK) : "memory");
    lds_barrier();
    StageRegs r0, r1;
    read_first(0, 0, r0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      spread(r0.pa[i]);
      r0.af[i] = convert(r0.pa[i][0], r0.pa[i][1]);
    }
    // Unrolled over the buffers (twice when their number is odd, so that the two fragment
    // register sets alternate consistently): whole rounds in one block of straight-line code, the
    // stages left over (fewer than a round) behind it.
    constexpr int UN = NS % 2 ? 2 * NS : NS;
    int kt = 0;
    for (; kt + UN <= nk; kt += UN) {
      static_for<UN>([&](auto U) {
        constexpr int u = decltype(U)::value;
        if constexpr (u % 2 == 0) stage(u % NS, kt + u, r0, r1);
        else stage(u % NS, kt + u, r1, r0);
      });
    }
    static_for<UN - 1>([&](auto U) {
      constexpr int u = decltype(U)::value;
      if (kt + u < nk) {
        if constexpr (u % 2 == 0) stage(u % NS, kt + u, r0, r1);
        else stage(u % NS, kt + u, r1, r0);
      }
    });
    // The loads beyond the range wrote zeros: they too are over before the buffers are reused.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] *= 0.5f;
  }
};

template <int WM, int WN, int TM, int TN, int NS = 4>
__global__ __launch_bounds__(256, 2) void spike_gemm_kernel(const GemmArgs a) {
  typedef SpikeTile<WM, WN, TM, TN, NS> Tile;
  constexpr int BM = Tile::BM, BN = Tile::BN, ST = Tile::ST, PI = Tile::PI, QI = Tile::QI;
  static_assert(NS * ST <= 81920, "two workgroups per compute unit");
  __shared__ __attribute__((aligned(16))) char lds[NS * ST];

  // An XCD gets a contiguous run of tiles (column tiles fastest): tiles sharing a row slab of
  // P share an L2.
  const int block = blockIdx.x;
  const int ntiles = a.tiles_m * a.tiles_n;
  const int tile = (block & 7) * ((ntiles + 7) >> 3) + (block >> 3);
  if (tile >= ntiles) return;
  const int row0 = (tile / a.tiles_n) * BM;
  const int col0 = (tile % a.tiles_n) * BN;
  const int nk = (a.kc + 31) >> 5;                           // stages

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int h = lane >> 5;
  const u32x4 rp = raw_rsrc(a.P, a.p_bytes), rq = raw_rsrc(a.Q, a.q_bytes);

  int pv[PI], qv[QI];
#pragma unroll
  for (int q = 0; q < PI; ++q) {
    const int row = Tile::p_row(wave, lane, q);
    pv[q] = row0 + row < a.rows ? (row0 + row) * a.ldp + Tile::p_unit(row, lane) * 16 : OOB;
  }
#pragma unroll
  for (int q = 0; q < QI; ++q) {
    const int row = Tile::q_row(wave, lane, q);
    qv[q] = ((col0 + row) * a.ldq + Tile::q_chunk(row, lane) * 8) * 2;
  }
  f32x16 acc[TM][TN];
  Tile::run(lds, rp, rq, pv, qv, nk, wave, lane, acc);

  // Epilogue.  The MFMAs take Q as their first operand, so a tile comes out transposed: the
  // lane holds row (lane & 31) of C and register r holds column 8*(r/4) + 4*(lane/32) + (r%4),
  // four consecutive columns per register quad.  The quads go to LDS (the stages are free
  // now; 16 rows of the tile fit one) and come back as whole rows, so that every store
  // instruction writes full, consecutive cache lines: row-per-register stores (two 128-byte
  // pieces per instruction) cost four times the instructions, and 16-byte stores straight
  // from the quads scatter 32-byte pieces over 32 rows, which slowed the loads of the
  // neighbouring workgroup.  The LDS row pitch of BN*4 + 16 bytes spreads the 16-byte writes
  // of 16 consecutive rows over all banks.
  static_assert(WM == 2 && WN == 2, "stage 2 wm + (row / 16) takes 16 rows");
  constexpr int CP = BN * 4 + 16;                     // bytes between rows of C in LDS
  static_assert(16 * CP <= ST, "16 rows of C fit a stage");
  constexpr int LPR = BN / 4;                         // lanes per row of the tile when storing
  constexpr int RPI = 64 / LPR;                       // rows per store instruction
  const rsrc_t rc = make_rsrc(a.C, (unsigned)((size_t)a.rows * a.ldc * 4));
  char *mine = lds + (2 * wm + ((lane >> 4) & 1)) * ST + (lane & 15) * CP;   // where this lane's quads go
  const char *from = lds + wave * ST;                                        // whose rows this wavefront stores
  const int srow = lane / LPR, scol = (lane % LPR) * 4;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        u32x4 v;
        v.x = __float_as_uint(acc[i][j][4 * q]);
        v.y = __float_as_uint(acc[i][j][4 * q + 1]);
        v.z = __float_as_uint(acc[i][j][4 * q + 2]);
        v.w = __float_as_uint(acc[i][j][4 * q + 3]);
        *(u32x4 *)(mine + ((wn * TN + j) * 32 + 8 * q + 4 * h) * 4) = v;
      }
    lds_barrier();
#pragma unroll
    for (int t = 0; t < 16; t += RPI) {
      const u32x4 v = *(const u32x4 *)(from + (srow + t) * CP + scol * 4);
      const int row = row0 + ((wave >> 1) * TM + i) * 32 + 16 * (wave & 1) + srow + t, col = col0 + scol;
      // Non-temporal: C is written once and read by a later kernel; kept out of the way, it
      // no longer evicts the P lines that the next stages (and the neighbouring column tiles)
      // are about to read again: 9 % (K = 1024) and 21 % (K = 700) on the whole kernel.
      const int vo = row < a.rows && col < a.ldc ? (row * a.ldc + col) * 4 : OOB;
      if (a.nt_store) __builtin_amdgcn_raw_buffer_store_b128(v, rc, vo, 0, NT);
      else __builtin_amdgcn_raw_buffer_store_b128(v, rc, vo, 0, 0);
    }
    if (i + 1 < TM) lds_barrier();                    // the rows are read before the next quads land
  }
}

template <int WM, int WN, int TM, int TN>
static hipError_t spike_gemm_launch(GemmArgs a, hipStream_t st) {
  dim3 grid(gemm_prepare<WM, WN, TM, TN>(a, 1), 1, 1);
  hipLaunchKernelGGL((spike_gemm_kernel<WM, WN, TM, TN>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace snn
