// Weight gradients dW = S^T dI on rounded-weight products, with the transposing LDS reads of
// gfx950: C[k][n] = sum_m S[m][k] G[m][n], contraction over the T*B rows m, the slow axis of both
// operands (S: 0/1 spike bytes [m][K]; G: current gradients, one dword per element holding a
// bfloat16 hi (low half) and lo (high half)).
//
// The general kernel (gemm.hpp) transposes 8 x 4 byte blocks and 8 x 2 word blocks in registers on
// their way to LDS: about 110 ALU instructions and 16 LDS writes per wavefront and 64 rows between its
// MFMAs, and it needs two workgroups per compute unit to hide them.  Here both operand tiles go from
// memory straight into LDS as they lie (buffer_load ... lds, the pipeline of the forward products), the
// few instructions left are dealt out one MFMA at a time (see `stage`), so one workgroup per compute
// unit multiplies as fast as two and the launch gets by with half the contraction splits, i.e. half
// the partial sums.  The fragments are read transposed:
//   ds_read_b64_tr_b8   the 16 lanes of a group each point at 8 bytes; the pieces of lanes 2r and
//                       2r + 1 form row r of an 8 x 16 byte matrix, and lane i receives column i:
//                       eight consecutive rows m of one spike column k - the A operand of
//                       v_mfma_f32_32x32x16_bf16 once the bytes are widened;
//   ds_read_b64_tr_b16  16 lanes each point at 8 bytes = four 16-bit elements; the pieces of lanes
//                       4e .. 4e + 3 form row e of a 4 x 16 matrix, lane i receives column i: four
//                       consecutive rows of one 16-bit column.  The words of G, read as a bfloat16
//                       matrix of twice the columns, give hi and lo of a neuron in adjacent columns of
//                       the B operand, hence in adjacent lanes of the accumulator: the two sums are
//                       kept apart over the whole contraction and joined by one cross-lane add at the
//                       end (smallest terms are never lost in a running sum of the large ones).
// A workgroup owns 128 rows k x 128 columns n of dW for one slice of the contraction (the splits
// and the order in which partial results are added are those of the general kernel); 2 x 2
// wavefronts hold 64 x 64 each, as 2 x 4 accumulator tiles (a column tile is 16 neurons x {hi, lo}).
// Stages of 32 rows m on three buffers: 4 KiB of S (rows of 128 bytes) and 16 KiB of G (rows of 128
// words) per stage; 16-byte units are placed at slot u ^ f(m) within a row (applied on the global
// side of the loads) so that the transposed reads, which touch 8 (S) or 4 (G) consecutive rows at
// the same columns, spread over the banks.
#pragma once
#include "gemm_stream.hpp"

namespace snn {

typedef int v2i32_t __attribute__((ext_vector_type(2)));
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v2i32_t *lds_v2i32_ptr;
typedef __attribute__((address_space(3))) v4i16_t *lds_v4i16_ptr;
typedef __attribute__((address_space(3))) char *lds_char_ptr;

template <int NS_>
struct WgradTr {
  static constexpr int BM = 128, BN = 128, MT = 32, NS = NS_;
  static constexpr int SP = MT * 128, GP = MT * 512, ST = SP + GP;   // bytes of a stage: S part, G part
  static constexpr int NL = 5;                                       // load instructions per wavefront and stage
  static constexpr int LDS_BYTES = NS * ST;
};

// PK: S is the raster packed along time (eight steps of a channel and sample in a byte, first step in
// the most significant bit), and the contraction runs in packed order: element m = 64 q + 8 mg + r is
// sample 8 bg + mg at step 8 tp + r for q = tp (B / 8) + bg.  The eight elements a lane feeds to an
// MFMA are then the eight bits of one byte: the S part of a stage is 4 samples x 128 bytes, read
// bytewise and expanded in registers; the rows of G are gathered in that order by the loads' per-lane
// offsets, so its tile in LDS and its fragment reads are those of the plain order.
template <bool PK, int NS>
__device__ __forceinline__ void wgrad_tr_body(const GemmArgs &a, const int block, char *lds) {
  typedef WgradTr<NS> G;
  constexpr int BM = G::BM, BN = G::BN, MT = G::MT;
  constexpr int SP = G::SP, ST = G::ST, NL = G::NL;
  // tile and split of this workgroup: as gemm_body
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
  const int nk = kend > kbeg ? (kend - kbeg + MT - 1) / MT : 0;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // Rows m from kend on read as zero: the buffers end there.  (PK: a split ends on a whole stage, and
  // the rows of G that belong to steps beyond T lie beyond its end.)
  const unsigned long long p_end = PK ? a.p_bytes : (unsigned long long)kend * a.ldp;
  const unsigned long long q_end = PK ? a.q_bytes : (unsigned long long)kend * a.ldq * 4ull;
  const u32x4 rp = raw_rsrc(a.P, (unsigned)(p_end < a.p_bytes ? p_end : a.p_bytes));
  const u32x4 rq = raw_rsrc(a.Q, (unsigned)(q_end < a.q_bytes ? q_end : a.q_bytes));
  const unsigned lds0 = (unsigned)(uintptr_t)(lds_ptr_t)lds;

  // Global side of the loads (the row offset of a stage is part of the lane's offset, which the
  // buffer's size bounds).  S: the wavefront's instruction fills rows 8 wave .. + 7 of the stage, lane
  // -> row lane / 8, slot lane % 8 holding unit slot ^ (row % 8).  G: instruction q fills rows
  // 2 (4 q + wave), + 1, lane -> row lane / 32, slot lane % 32 holding unit slot ^ 4 (row % 4).
  // PK: S rows are the stage's four samples (lanes 0..31 of wavefront 0 fetch them, natural order);
  // stage row rr of G is sample rr / 8 of the four at step rr % 8 of the eight: B rows apart per step.
  int pv, qv[4];
  int pk_tp = 0, pk_rem = 0;                           // PK: the next stage to issue starts at packed row pk_tp B + pk_rem
  if constexpr (PK) {
    pk_tp = (kbeg >> 3) / a.pk_B;
    pk_rem = (kbeg >> 3) - pk_tp * a.pk_B;
    pv = wave == 0 && lane < 32 ? (lane >> 3) * a.ldp + row0 + 16 * (lane & 7) : OOB;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int rr = 2 * (4 * q + wave) + (lane >> 5), uu = (lane & 31) ^ (4 * (rr & 3));
      qv[q] = (((rr & 7) * a.pk_B + (rr >> 3)) * a.ldq + col0 + 4 * uu) * 4;
    }
  } else {
    const int r = 8 * wave + (lane >> 3), u = (lane & 7) ^ (r & 7);
    pv = (kbeg + r) * a.ldp + row0 + 16 * u;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int rr = 2 * (4 * q + wave) + (lane >> 5), uu = (lane & 31) ^ (4 * (rr & 3));
      qv[q] = ((kbeg + rr) * a.ldq + col0 + 4 * uu) * 4;
    }
  }
  const int pstep = MT * a.ldp, qstep = MT * a.ldq * 4;
  struct Issue {
    u32x4 p, q;
    unsigned dst;
    int pbase, qbase;                                  // PK: byte offsets of the stage in S and G
  };
  auto issue_prepare = [&](int kt_any, int buf) {
    const int kt = __builtin_amdgcn_readfirstlane(kt_any);
    Issue r;
    r.p = rp; r.q = rq;
    if (kt >= nk) r.p.z = r.q.z = 0;                   // beyond the contraction: same instruction count, nothing fetched
    r.dst = __builtin_amdgcn_readfirstlane(lds0 + buf * ST + 1024 * wave);
    r.pbase = r.qbase = 0;
    if constexpr (PK) {
      r.pbase = __builtin_amdgcn_readfirstlane((pk_tp * a.pk_B + pk_rem) * a.ldp);
      r.qbase = __builtin_amdgcn_readfirstlane((8 * pk_tp * a.pk_B + pk_rem) * a.ldq * 4);
      pk_rem += 4;
      if (pk_rem >= a.pk_B) { pk_rem = 0; ++pk_tp; }
    }
    return r;
  };
  auto issue_load = [&](const Issue &r, auto N) {
    constexpr int n = decltype(N)::value;
    if constexpr (PK) {
      if constexpr (n == 0) load_to_lds_b128(r.p, r.dst, pv == OOB ? OOB : pv + r.pbase, 0);
      else load_to_lds_b128(r.q, r.dst + SP + 4096 * (n - 1), qv[n - 1] + r.qbase, 0);
    } else if constexpr (n == 0) {
      load_to_lds_b128(r.p, r.dst, pv, 0);
      pv += pstep;
    } else {
      load_to_lds_b128(r.q, r.dst + SP + 4096 * (n - 1), qv[n - 1], 0);
      qv[n - 1] += qstep;
    }
  };
  auto issue = [&](int kt_any, int buf) {
    const Issue r = issue_prepare(kt_any, buf);
    static_for<NL>([&](auto N) { issue_load(r, N); });
  };

  // LDS side.  A lane belongs to group g = lane / 16 with index j in it.
  // A (tr_b8), MFMA step s, row tile i: the lane points at stage row 16 s + 8 (g / 2) + j / 2 of S, bytes
  // 64 wm + 32 i + 16 (g % 2) + 8 (j % 2) .. + 7.
  // B (tr_b16), step s, half e2, column tile t: stage row 16 s + 8 (g / 2) + 4 e2 + j / 4 of G, words
  // 64 wn + 16 t + 8 (g % 2) + 2 (j % 4), + 1.
  // Step, half and stage only add constants to the address (they leave row % 8 and row % 4 alone).
  // PK, A: the byte of sample 2 s + lane / 32 of the stage's four and channel 64 wm + 32 i + lane % 32.
  const int g = lane >> 4, j = lane & 15;
  lds_char_ptr fa[2], fb[4];
  {
    lds_char_ptr base = (lds_char_ptr)lds;
    const int ra = 8 * (g >> 1) + (j >> 1), rb = 8 * (g >> 1) + (j >> 2);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fa[i] = PK ? base + (lane >> 5) * 128 + 64 * wm + 32 * i + (lane & 31)
                 : base + ra * 128 + (((4 * wm + 2 * i + (g & 1)) ^ (ra & 7)) << 4) + 8 * (j & 1);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      fb[t] = base + SP + rb * 512 + ((16 * wn + 4 * (t ^ (rb & 3)) + 2 * (g & 1) + ((j >> 1) & 1)) << 4) + 8 * (j & 1);
  }

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.f;

  auto convert = [&](v2i32_t x) {                      // eight 0/1 bytes (PK: the eight bits of x.x) -> eight bfloat16 of value 2 x spike
    u32x4 d;
    if constexpr (PK) {
      // z holds the byte at bits 0..7 and again at bits 17..24: shifted left by 7 + 2 j, bit 14 is step
      // 2 j and bit 30 is step 2 j + 1
      const uint32_t z = (uint32_t)x.x | ((uint32_t)x.x << 17);
      d.x = (z << 7) & 0x40004000u;
      d.y = (z << 9) & 0x40004000u;
      d.z = (z << 11) & 0x40004000u;
      d.w = (z << 13) & 0x40004000u;
      return __builtin_bit_cast(bf16x8, d);
    }
    const uint32_t t0 = (uint32_t)x.x << 6, t1 = (uint32_t)x.y << 6;
    d.x = __builtin_amdgcn_perm(0u, t0, 0x010C000Cu);
    d.y = __builtin_amdgcn_perm(0u, t0, 0x030C020Cu);
    d.z = __builtin_amdgcn_perm(0u, t1, 0x010C000Cu);
    d.w = __builtin_amdgcn_perm(0u, t1, 0x030C020Cu);
    return __builtin_bit_cast(bf16x8, d);
  };

  // One stage in buffer u.  At its barrier every wavefront has seen its own loads of the stage land
  // and has left stage kt - 1, whose buffer takes the loads of stage kt + NS - 1.
  //
  // Measured with one wavefront per SIMD: whatever sits between two MFMAs beyond the 32 cycles the
  // first one keeps the matrix unit is lost (fragment reads, conversions and load issue in blocks of
  // their own: 1065 cycles per stage for 512 cycles of MFMA).  The order is therefore fixed by hand
  // (scheduling barriers), one MFMA per slot followed by a small share of the stage's other
  // instructions.  The eight MFMAs of a stage's second step are carried over the next barrier in
  // registers (slots 0..7), so that the fragment reads of the first step, issued in slots 0..3, are
  // back before their use in slot 8; the reads of the second step follow in slots 8..11.
  struct Pending {
    bf16x8 af[2], bq[4];
  };
  auto read_a = [&](auto U, auto S, v2i32_t (&ar)[2]) {
    constexpr int off = decltype(U)::value * ST + decltype(S)::value * (PK ? 256 : 2048);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if constexpr (PK) {
        ar[i].x = *(const __attribute__((address_space(3))) unsigned char *)(fa[i] + off);
        ar[i].y = 0;
      } else {
        ar[i] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i32_ptr)(fa[i] + off));
      }
    }
  };
  auto read_b = [&](auto U, auto S, int t, bf16x8 &bq) {
    constexpr int off = decltype(U)::value * ST + decltype(S)::value * 8192;
    const v2i32_t k03 = __builtin_bit_cast(v2i32_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(fb[t] + off)));
    const v2i32_t k47 = __builtin_bit_cast(v2i32_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(fb[t] + (off + 2048))));
    u32x4 w;
    w.x = (uint32_t)k03.x; w.y = (uint32_t)k03.y; w.z = (uint32_t)k47.x; w.w = (uint32_t)k47.y;
    bq = __builtin_bit_cast(bf16x8, w);
  };
  auto mfma = [&](const Pending &x, int t, int i) {
    acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.af[i], x.bq[t], acc[i][t], 0, 0, 0);
  };
  auto multiply = [&](const Pending &x) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < 2; ++i) mfma(x, t, i);
  };
  typedef std::integral_constant<int, 0> I0;
  typedef std::integral_constant<int, 1> I1;
  typedef std::integral_constant<int, 2> I2;
  typedef std::integral_constant<int, 3> I3;
  typedef std::integral_constant<int, 4> I4;
#define SNN_SLOT_END __builtin_amdgcn_sched_barrier(0)
  auto stage = [&](auto U, int kt, Pending &pend) {
    constexpr int u = decltype(U)::value;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NL) : "memory");
    lds_barrier();
    SNN_SLOT_END;
    Pending now;
    v2i32_t ar0[2], ar1[2];
    const Issue ld = issue_prepare(kt + NS - 1, (u + NS - 1) % NS);
    mfma(pend, 0, 0); read_a(U, I0(), ar0); read_b(U, I0(), 0, now.bq[0]); SNN_SLOT_END;
    mfma(pend, 0, 1); read_b(U, I0(), 1, now.bq[1]); issue_load(ld, I0()); SNN_SLOT_END;
    mfma(pend, 1, 0); read_b(U, I0(), 2, now.bq[2]); issue_load(ld, I1()); SNN_SLOT_END;
    mfma(pend, 1, 1); read_b(U, I0(), 3, now.bq[3]); issue_load(ld, I2()); SNN_SLOT_END;
    mfma(pend, 2, 0); issue_load(ld, I3()); SNN_SLOT_END;
    mfma(pend, 2, 1); issue_load(ld, I4()); SNN_SLOT_END;
    mfma(pend, 3, 0); now.af[0] = convert(ar0[0]); SNN_SLOT_END;
    mfma(pend, 3, 1); now.af[1] = convert(ar0[1]); SNN_SLOT_END;
    mfma(now, 0, 0); read_a(U, I1(), ar1); read_b(U, I1(), 0, pend.bq[0]); SNN_SLOT_END;
    mfma(now, 0, 1); read_b(U, I1(), 1, pend.bq[1]); SNN_SLOT_END;
    mfma(now, 1, 0); read_b(U, I1(), 2, pend.bq[2]); SNN_SLOT_END;
    mfma(now, 1, 1); read_b(U, I1(), 3, pend.bq[3]); SNN_SLOT_END;
    mfma(now, 2, 0); SNN_SLOT_END;
    mfma(now, 2, 1); SNN_SLOT_END;
    mfma(now, 3, 0); pend.af[0] = convert(ar1[0]); SNN_SLOT_END;
    mfma(now, 3, 1); pend.af[1] = convert(ar1[1]); SNN_SLOT_END;
  };
#undef SNN_SLOT_END

#pragma unroll
  for (int t = 0; t < NS - 1; ++t) issue(t, t);
  Pending pend;                                         // zeros in front of the first stage
  {
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 2; ++i) pend.af[i] = __builtin_bit_cast(bf16x8, z);
#pragma unroll
    for (int t = 0; t < 4; ++t) pend.bq[t] = __builtin_bit_cast(bf16x8, z);
  }
  // whole rounds of NS stages as straight-line code (the accumulators keep their registers), then the rest
  int kt = 0;
  for (; kt + NS <= nk; kt += NS) {
    static_for<NS>([&](auto U) { stage(U, kt + decltype(U)::value, pend); });
  }
  static_for<NS - 1>([&](auto U) {
    if (kt + decltype(U)::value < nk) stage(U, kt + decltype(U)::value, pend);
  });
  multiply(pend);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // Accumulator layout of the 32x32 MFMA: lane holds column (lane & 31) of the tile - neuron
  // (lane & 31) / 2, hi in even lanes and lo in odd ones; register r holds row 8 (r / 4) + 4 (lane / 32)
  // + (r % 4).  hi + lo by a cross-lane add; then even lanes store column tile t and odd lanes
  // column tile t + 1 (both lanes of a pair hold both sums).  The spikes entered as 2.0: halved here.
  float *C = a.C + (size_t)split * a.c_split_stride;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int tp = 0; tp < 4; tp += 2)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float x0 = acc[i][tp][r], x1 = acc[i][tp + 1][r];
        const float s0 = x0 + __shfl_xor(x0, 1), s1 = x1 + __shfl_xor(x1, 1);
        const float v = 0.5f * ((lane & 1) ? s1 : s0);
        const int row = row0 + 64 * wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int col = col0 + 64 * wn + 16 * (tp + (lane & 1)) + ((lane & 31) >> 1);
        if (row < a.rows && col < a.cols) {
          const size_t o = (size_t)row * a.ldc + col;
          if (a.nt_store) __builtin_nontemporal_store(v, &C[o]);
          else C[o] = v;
        }
      }
}

// The weight-gradient jobs of wide layers (rounded weights); a job's S may be the raster packed along time.
// NS: stages in flight.  3 (60 KiB) lets two workgroups share a compute unit.  More do not help, not even
// a launch of one workgroup per compute unit (700-128-128-20, T*B = 32768, 256 workgroups: 18.1 us with
// 3, 18.3 with 4, 19.6 with 6): the latency of the loads is covered.
template <int NS>
__global__ __launch_bounds__(256, 2) void wgrad_tr_jobs_kernel(const GemmJobs jobs) {
  static_assert(WgradTr<NS>::LDS_BYTES <= 163840, "LDS of a compute unit");
  __shared__ __attribute__((aligned(16))) char lds[WgradTr<NS>::LDS_BYTES];
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first_block[j + 1]) ++j;
  if (jobs.job[j].packed) wgrad_tr_body<true, NS>(jobs.job[j], blockIdx.x - jobs.first_block[j], lds);
  else wgrad_tr_body<false, NS>(jobs.job[j], blockIdx.x - jobs.first_block[j], lds);
}

static hipError_t wgrad_tr_jobs_launch(const GemmJobs &jobs, hipStream_t st) {
  if (jobs.njobs == 0) return hipSuccess;
  dim3 grid(jobs.first_block[jobs.njobs], 1, 1);
  hipLaunchKernelGGL(wgrad_tr_jobs_kernel<3>, grid, dim3(256), 0, st, jobs);
  return hipGetLastError();
}

}  // namespace snn
