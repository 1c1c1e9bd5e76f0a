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
//   * three or four LDS stages of 64 or 32 contraction elements and one barrier per stage, at its
//     start: behind it the loads of stage t + NS - 1 are issued into the buffer stage t - 1 has
//     left, so a load has NS - 2 stages to land (the P operand comes from HBM on first touch);
//   * the last MFMA step of a stage is carried over the next stage's barrier (its operands are in
//     registers) and covers the arrival of that stage's first fragments.
//
// Contraction order inside a stage.  A lane holds 8 consecutive k per MFMA.  Reading a lane's
// P bytes 16 at a time (two steps' worth) fixes which k a step covers: with SPS steps per stage,
// step s of lane half h = lane/32 covers k = 8 SPS h + 8s .. +7, and the Q fragment of that step is
// read from the matching 16-byte chunk SPS h + s of the row.
//
// Tails.  Rows of P beyond the product read as zero (lane offset beyond the buffer).  Along
// k nothing is masked on the P side: Q is zero-padded to a multiple of 64 along k, and
// whatever P yields there (bytes of the next row, 0 or 1 like all others) meets those zeros.
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
// bytes; qv: Q, bfloat16), takes the stages through `lds` (lds_bytes(pk) bytes) and leaves the
// products in acc; on return every load has landed and every wavefront is past its last
// fragment read, so the caller may reuse the LDS.
//
// KS: contraction elements per stage, 32 or 64.  What a stage costs a compute unit is the number of
// cache lines its loads touch, not their bytes (a line per clock through the L1, and every line is
// a miss): a stage of 64 brings 64-byte pieces of the spike rows and whole 128-byte lines of the
// weight rows where a stage of 32 brings 32- and 64-byte pieces of the same lines twice.  Loads
// alone, on this pipeline (128 x 128 tile, K = 700, one workgroup per compute unit): 660 cycles per
// 32 contraction elements with stages of 32, 486 with stages of 64.
template <int WM, int WN, int TM, int TN, int NS, int KS = 64>
struct SpikeTile {
  static_assert(WM * WN == 4, "four wavefronts per workgroup");
  static_assert(KS == 32 || KS == 64, "stages of 32 or 64 contraction elements");
  static constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  static constexpr int KSTAGE = KS;
  static constexpr int SPS = KS / 16;                 // MFMA steps per stage
  static constexpr int PU = KS / 16, QC = KS / 8;     // 16-byte units per row of P, chunks per row of Q, in a stage
  static constexpr int UPL = KS / 32;                 // units of its row a lane reads per stage (8 bytes per step)
  // (a tile of few rows still gives P a whole KiB per wavefront and stage: the rows beyond the tile
  // are loaded as rows outside the product, i.e. as zeros, and never read)
  static constexpr int PROWS = BM * KS < 4096 ? 4096 / KS : BM;
  static constexpr int PT = PROWS * KS, QT = BN * 2 * KS, ST = PT + QT;   // bytes: P part, Q part, stage
  static constexpr int PI = PT / 4096, QI = QT / 4096;                    // load instructions per wavefront and stage
  static constexpr int NL = PI + QI;
  static_assert(PT % 4096 == 0 && QT % 4096 == 0, "whole KiB per wavefront");
  static_assert(NS >= 3, "a stage in use, one landing, one being asked for");
  typedef u32x4 frag_t;
  // Packed P operand: the whole block of the sample (BM / 8 packed rows of up to 1024 bytes) sits
  // in LDS for all stages, ahead of the stages, which then hold Q alone.  A row pitch of 1088 bytes
  // puts the four packed rows a fragment read touches on different banks.
  static constexpr int PKP = 1088, PKB = ((BM / 8) * PKP + 1023) / 1024 * 1024;   // (the stages behind it start on a KiB)
  static constexpr int lds_bytes(bool pk) { return pk ? PKB + NS * QT : NS * ST; }

  // Where a row's 16-byte pieces sit inside the row in LDS: piece c of row r at slot c ^ swz(r), so
  // that the fragment reads (32 consecutive rows, the same piece) touch every bank equally: the LDS
  // takes a 16-byte read 16 lanes at a time over its 64 banks, so among 16 consecutive rows those
  // that start on the same bank (every 256 / row bytes-th) must differ in their slot.  (Rows of 128
  // bytes with slot c ^ (r % 8) measured 48 conflict cycles per stage and wavefront.)
  static __device__ __forceinline__ int swz_p(int r) { return KS == 32 ? (r >> 3) & 1 : (r >> 2) & 3; }
  static __device__ __forceinline__ int swz_q(int r) { return KS == 32 ? (r >> 2) & 3 : (r >> 1) & 7; }
  // Global side of the loads: a wavefront's 64 lanes fill 1 KiB of consecutive LDS, so the
  // permutation is applied here: each lane fetches the piece that belongs at its slot.  P
  // instruction q of a wavefront fills rows (1024 / KS)(wave + 4 q) .. of the stage, KS bytes each:
  // lane -> row lane / PU, slot lane % PU.  Q instruction q fills rows (512 / KS)(wave + 4 q) ..,
  // 2 KS bytes each: lane -> row lane / QC, slot lane % QC.
  static __device__ __forceinline__ int p_row(int wave, int lane, int q) { return (1024 / KS) * (wave + 4 * q) + lane / PU; }
  static __device__ __forceinline__ int p_unit(int row, int lane) { return (lane % PU) ^ swz_p(row); }
  static __device__ __forceinline__ int q_row(int wave, int lane, int q) { return (512 / KS) * (wave + 4 * q) + lane / QC; }
  static __device__ __forceinline__ int q_chunk(int row, int lane) { return (lane % QC) ^ swz_q(row); }

  // PK: P comes from `pk` (packed along time; BM rows = time steps of one sample) instead of rp /
  // pv: a lane's KS / 2 bytes of row r, columns (KS / 2) h .. of a stage, are bit 7 - r % 8 of the
  // packed bytes at packed row r / 8; no P loads per stage.
  template <bool PK = false>
  static __device__ __forceinline__ void run(char *lds, const u32x4 rp, const u32x4 rq, const int (&pv)[PI],
                                             const int (&qv)[QI], const int nk, const int wave, const int lane,
                                             f32x16 (&acc)[TM][TN], const PackedRows *pk = nullptr) {
    const int wm = wave / WN, wn = wave % WN;
    constexpr int STQ = PK ? QT : ST;               // bytes of a stage
    constexpr int QOFF = PK ? 0 : PT;               // where Q starts inside a stage
    constexpr int PIK = PK ? 0 : PI;                // P load instructions per wavefront and stage
    constexpr int NLK = PIK + QI;                   // load instructions per wavefront and stage
    constexpr int M = TM * TN;                      // MFMAs per step
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
      return r;
    };
    auto issue_load = [&](const IssueRegs &r, int n) {        // load instruction n of the stage (P first)
      if (n < PIK) load_to_lds_b128(r.p, r.dst + 4096 * n, pv[n < PI ? n : 0], r.kt * KS);
      else load_to_lds_b128(r.q, r.dst + QOFF + 4096 * (n - PIK), qv[n - PIK], r.kt * 2 * KS);
    };
    auto issue = [&](int kt_any, int buf) {
      const IssueRegs r = issue_prepare(kt_any, buf);
#pragma unroll
      for (int n = 0; n < NLK; ++n) issue_load(r, n);
    };

    // LDS side of the fragment reads: lane half h = lane / 32 reads the UPL units UPL h .. of its P
    // row (8 bytes per MFMA step: step s of a stage covers k = (KS / 2) h + 8 s .. + 7) and, for
    // step s, chunk SPS h + s of its Q row.  Rows 32 apart share the permutation.
    const int h = lane >> 5;
    int fa[UPL], fb[SPS];
    {
      const int ra = wm * TM * 32 + (lane & 31), rb = wn * TN * 32 + (lane & 31);
#pragma unroll
      for (int e = 0; e < UPL; ++e)
        fa[e] = PK ? (ra >> 3) * PKP + (KS / 2) * h + 16 * e : ra * KS + (((UPL * h + e) ^ swz_p(ra)) << 4);
#pragma unroll
      for (int st = 0; st < SPS; ++st) fb[st] = QOFF + rb * 2 * KS + (((SPS * h + st) ^ swz_q(rb)) << 4);
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

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
      u32x4 x = d;
      asm volatile("" : "+v"(x));                             // the fragment is formed here, not next to its use
      return __builtin_bit_cast(bf16x8, x);
    };
    // Operands of a stage's last MFMA step: issued behind the next stage's barrier (they are in
    // registers), so that the matrix units have work while that stage's first fragments arrive.
    struct Pending {
      frag_t q[TN];
      bf16x8 af[TM];
    };
    // One stage in buffer u.  At its barrier every wavefront has seen its own loads of the stage
    // land (so the buffer is complete) and has left stage kt - 1, whose buffer, u + NS - 1, takes the
    // loads of stage kt + NS - 1.
    //
    // One wavefront per SIMD: nothing but this wavefront's own independent instructions fills the
    // 32 cycles an MFMA keeps the matrix unit.  The order is therefore fixed by hand (scheduling
    // barriers): behind the barrier the fragment reads and the load issue, then the previous
    // stage's last step, and from there one MFMA, then the few conversion instructions of a fragment
    // needed a step later.  Left to the scheduler, the conversions of a whole stage sit in front of
    // its first MFMA and the fragment reads next to their use, each followed by its wait.
    auto stage = [&](int u, int kt, Pending &pend) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NLK) : "memory");   // younger stages may still be in flight
      lds_barrier();
      const char *st = stages + u * STQ;
      frag_t pa[TM][UPL], q[2][TN];
      bf16x8 af[2][TM];
      auto read_p = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int e = 0; e < UPL; ++e)
            pa[i][e] = PK ? *(const frag_t *)(lds + fa[e] + i * 4 * PKP + kt * KS) : *(const frag_t *)(st + fa[e] + i * 32 * KS);
      };
      auto read_q = [&](int sp) {
#pragma unroll
        for (int j = 0; j < TN; ++j) q[sp & 1][j] = *(const frag_t *)(st + fb[sp] + j * 64 * KS);
      };
      auto conv = [&](int sp, int i) {                  // the P fragment of row tile i for step sp
        af[sp & 1][i] = convert(pa[i][sp >> 1][2 * (sp & 1)], pa[i][sp >> 1][2 * (sp & 1) + 1]);
      };
      if constexpr (TM == 2 && TN == 2 && KS == 64) {
        // 16 MFMAs: the step left over from the stage before (operands in registers), then steps 0 to
        // 2; behind MFMA k the work of slot k, at most about seven instructions each.
        IssueRegs ir;
        static_for<16>([&](auto K) {
          constexpr int k = decltype(K)::value, sp = k / 4 - 1, i = (k % 4) / 2, j = k % 2;
          if constexpr (k < 4) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pend.q[j]), pend.af[i], acc[i][j], 0, 0, 0);
          else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q[sp & 1][j]), af[sp & 1][i], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (k == 0) { read_p(); read_q(0); }
          if constexpr (k == 1) { ir = issue_prepare(kt + NS - 1, (u + NS - 1) % NS); issue_load(ir, 0); }
          if constexpr (k == 2) { issue_load(ir, 1); if (NLK > 2) issue_load(ir, 2); }
          if constexpr (k == 3) { spread(pa[0][0]); conv(0, 0); }
          if constexpr (k == 4) { spread(pa[1][0]); conv(0, 1); }
          if constexpr (k == 5) { if (NLK > 3) issue_load(ir, 3); read_q(1); }
          if constexpr (k == 6) { conv(1, 0); if (NLK > 4) issue_load(ir, 4); }
          if constexpr (k == 7) { conv(1, 1); if (NLK > 5) issue_load(ir, 5); }
          if constexpr (k == 8) { read_q(2); spread(pa[0][1]); }
          if constexpr (k == 9) conv(2, 0);
          if constexpr (k == 10) { spread(pa[1][1]); conv(2, 1); }
          if constexpr (k == 11) read_q(3);
          if constexpr (k == 12) conv(3, 0);
          if constexpr (k == 13) conv(3, 1);
          __builtin_amdgcn_sched_barrier(0);
        });
        static_assert(NLK <= 6, "slots for six load instructions");
      } else {
        read_p();
        read_q(0);
        __builtin_amdgcn_sched_barrier(0);
        issue(kt + NS - 1, (u + NS - 1) % NS);
        __builtin_amdgcn_sched_barrier(0);
        // the step left over from the stage before, with this stage's first conversions behind its MFMAs
        static_for<M>([&](auto X) {
          constexpr int x = decltype(X)::value, i = x / TN, j = x % TN;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pend.q[j]), pend.af[i], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (x < TM) {
#pragma unroll
            for (int e = 0; e < UPL; ++e) spread(pa[x][e]);
            conv(0, x);
          }
          __builtin_amdgcn_sched_barrier(0);
        });
        static_for<SPS - 1>([&](auto S) {
          constexpr int sp = decltype(S)::value;          // this step; the fragments of step sp + 1 are formed under it
          read_q(sp + 1);
          __builtin_amdgcn_sched_barrier(0);
          static_for<M>([&](auto X) {
            constexpr int x = decltype(X)::value, i = x / TN, j = x % TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q[sp & 1][j]), af[sp & 1][i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (x < TM) conv(sp + 1, x);
            __builtin_amdgcn_sched_barrier(0);
          });
        });
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) pend.q[j] = q[(SPS - 1) & 1][j];
#pragma unroll
      for (int i = 0; i < TM; ++i) pend.af[i] = af[(SPS - 1) & 1][i];
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
    Pending pend;                                     // nothing is left over before the first stage: zeros
#pragma unroll
    for (int j = 0; j < TN; ++j) pend.q[j] = frag_t{0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < TM; ++i) pend.af[i] = __builtin_bit_cast(bf16x8, frag_t{0u, 0u, 0u, 0u});
    // Unrolled over the buffers: whole rounds in one block of straight-line code, the stages left
    // over (fewer than a round) behind it.
    int kt = 0;
    for (; kt + NS <= nk; kt += NS) {
      static_for<NS>([&](auto U) {
        constexpr int u = decltype(U)::value;
        stage(u, kt + u, pend);
      });
    }
    static_for<NS - 1>([&](auto U) {
      constexpr int u = decltype(U)::value;
      if (kt + u < nk) stage(u, kt + u, pend);
    });
    static_for<M>([&](auto X) {                        // the last stage's last step
      constexpr int x = decltype(X)::value, i = x / TN, j = x % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pend.q[j]), pend.af[i], acc[i][j], 0, 0, 0);
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
  typedef SpikeTile<WM, WN, TM, TN, NS, 32> Tile;     // (stages of 64 would leave this tile two buffers)
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
