// C ABI of the library (see include/snn.h): context, workspace carve-up, the layer loops of
// the forward and reverse passes, and the launches.  Host code only enqueues kernels; every
// step of the path runs on the GPU.
#include "../../include/snn.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "gemm.hpp"
#include "gemm_stream.hpp"
#include "wgrad_tr.hpp"
#include "layer_forward.hpp"
#include "scan.hpp"
#include "layer_reverse.hpp"
#include "rlif.hpp"
#include "rlif_persist.hpp"

using namespace snn;

// Scratch of snn_weight_grad_static: the per-split partial sums of one weight-gradient product.
// One copy per GPU, held from the moment the library is loaded on it until the process ends.
// Host code never uses this name as an address: it asks for the device address once per device
// (static_scratch) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[SNN_STATIC_SCRATCH_BYTES];

namespace {

inline size_t rup(size_t x, size_t m) { return (x + m - 1) / m * m; }

struct Layer {
  int K = 0, N = 0;        // fan-in, fan-out
  int ld = 0;              // padded fan-out of the activation tensors (multiple of 8)
  bool recurrent = false, spiking = false;
  bool adaptive = false;   // adaptive firing threshold: theta + A_t, A' = gamma A + kappa S
  float gamma = 0.f, kappa = 0.f;
  float *A = nullptr;      // [M][ld] adaptation in force at each step (adaptive layers only)
  float beta = 0.f;        // initial decay of the layer (config); the live values are beta_v
  float *beta_v = nullptr; // [ld] one decay per neuron / class (padding 0)
  float *dbeta = nullptr;  // [ld] gradient of the decays (only with learn_beta)
  float *part_b = nullptr; // [B][ld] per-sample parts of dbeta
  float *Wm = nullptr, *dW = nullptr;
  uint16_t *Qf = nullptr, *Qb = nullptr;       // [plane][N pad 128][K pad 64], [plane][K pad 128][N pad 64]
  int ldqf = 0, ldqb = 0;
  long long qf_plane = 0, qb_plane = 0;
  float *Rm = nullptr, *dR = nullptr;
  uint16_t *QRf = nullptr, *QRb = nullptr;     // [plane][to][from], [plane][from][to]
  int ldqr = 0;
  long long qr_plane = 0;
  float *I = nullptr, *V = nullptr, *dS = nullptr;   // [M][ld]; readout: I = J, V = Y
  uint8_t *S = nullptr;
  uint32_t *dI = nullptr;                             // [M][ld] fp32 bits or HL; readout: dJ
  float *g[2] = {nullptr, nullptr};                   // recurrent reverse state [B][ld]
  void *rp_space = nullptr;                           // exchange space of the one-launch forward loop of a wide recurrent layer
  bool i_ready = true;     // I is in memory (false: the last forward pass ran the layer in one launch and never stored it)
  bool ds_ready = true;    // dS is in memory (false: the layer's reverse scan formed it itself in the last backward pass)
  int splits_w = 1, splits_r = 1;                     // contraction splits of dW and dR
  long long per_w = 0, per_r = 0;                     // rows per split
  float *part_w = nullptr, *part_r = nullptr;         // per-split partial results
};

struct Prof {
  int cls = SNN_K_NONE, layer = 0;
  std::vector<hipEvent_t> ev;     // start/stop pairs
  size_t used = 0;
  int every = 1;                  // bracket every n-th matching launch
  long long seen = 0;             // matching launches since the last select
};

}  // namespace

struct snn_ctx {
  int T = 0, B = 0, L = 0;
  long long M = 0;
  std::vector<int> sizes;
  std::vector<Layer> layers;      // index 0..L-1  (text layer l = index + 1)
  float theta = 1.f, slope = 1.f;
  int surrogate = 0, precision = 0, nplanes = 1;
  bool hl = false;                // current gradients held in hi/lo form
  int C = 0, ldC = 0;
  float *z = nullptr, *dz = nullptr, *loss_b = nullptr, *loss = nullptr;
  int *tstar = nullptr, *err_flag = nullptr;
  char *ws = nullptr;
  size_t ws_bytes = 0;
  hipStream_t stream = nullptr;
  int state = 0;                  // 0 fresh, 1 forward done, 2 backward done
  bool dj_ready = false;          // the fused readout kernel has already written dJ
  bool loss_ready = false;        // the mean of loss_b has been taken since the last readout
  int wall_khz = 100000;          // rate of the device's constant clock
  int cus = 0;                    // compute units of the device
  bool wg_tall = false;           // weight-gradient products use 256 x 128 tiles
  bool integral = false;          // integral cross-entropy instead of max over time
  bool learn_beta = false;        // decays are trained: dbeta in snn_backward, clipped update in snn_sgd_step
  const uint8_t *x_eff = nullptr;  // raster the products read: the caller's, or x_buf
  uint8_t *x_buf = nullptr;        // [T*B][ldx]: zero-padded copy (N_0 not a multiple of 4) or unpacked input
  bool x_padded = false;           // the caller's raster must be copied into x_buf
  const uint8_t *x_packed = nullptr;  // the caller's raster packed along time (snn_forward_packed)
  bool x_direct = false;           // layer 1's launches read x_packed themselves; x_eff exists only once x_unpacked
  bool x_unpacked = false;
  int ldx = 0;                     // row length of x_eff
  const int32_t *labels_dev = nullptr;
  ReduceJobs pending;             // partial sums of the last backward pass that have not been added yet
  bool reduce_pending = false;
  int opt[SNN_OPT_COUNT] = {4, 1, 1, 1, 1, 0, 128, 1024, 128, 1, 0, 0, 1, 1, 18, 0};   // snn_option values, in the enum's order
  uint32_t *hand = nullptr;       // hand-over space of the forward launches that give a sample to two workgroups
  int hand_parts = 1;             // hand-over regions per sample (one per column block of a layer)
  int fwd_epoch = 0;              // number of such launches so far (their flags count from epoch * 1024)
  std::string err;
  Prof prof;
};

namespace {

thread_local std::string g_err;   // errors of calls that have no context

int fail(snn_ctx *c, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_err = buf;
  return code;
}

#define HIPCHK(c, call)                                                                     \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail((c), SNN_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),  \
                  __FILE__, __LINE__);                                                      \
  } while (0)

int validate(const snn_config *cfg) {
  if (!cfg) return fail(nullptr, SNN_ERR_NULL, "config is NULL");
  if (!cfg->sizes || !cfg->beta) return fail(nullptr, SNN_ERR_NULL, "config.sizes / config.beta is NULL");
  if (cfg->T <= 0 || cfg->B <= 0) return fail(nullptr, SNN_ERR_ARG, "T and B must be positive");
  if (cfg->n_layers < 2 || cfg->n_layers > SNN_MAX_LAYERS)
    return fail(nullptr, SNN_ERR_ARG, "n_layers must be in [2, %d] (at least one spiking layer and the readout)",
                SNN_MAX_LAYERS);
  for (int i = 0; i <= cfg->n_layers; ++i)
    if (cfg->sizes[i] <= 0 || cfg->sizes[i] > (1 << 20)) return fail(nullptr, SNN_ERR_ARG, "sizes[%d] out of range", i);
  for (int i = 0; i < cfg->n_layers; ++i)
    if (!(cfg->beta[i] >= 0.f && cfg->beta[i] <= 1.f)) return fail(nullptr, SNN_ERR_ARG, "beta[%d] outside [0,1]", i);
  if (!(cfg->threshold > 0.f)) return fail(nullptr, SNN_ERR_ARG, "threshold must be positive");
  if (!(cfg->slope > 0.f)) return fail(nullptr, SNN_ERR_ARG, "slope must be positive");
  if (cfg->surrogate < 0 || cfg->surrogate > 5) return fail(nullptr, SNN_ERR_ARG, "unknown surrogate");
  if (cfg->precision < 0 || cfg->precision > 1) return fail(nullptr, SNN_ERR_ARG, "unknown precision");
  if (cfg->loss < 0 || cfg->loss > 1) return fail(nullptr, SNN_ERR_ARG, "unknown loss");
  if (cfg->learn_beta < 0 || cfg->learn_beta > 1) return fail(nullptr, SNN_ERR_ARG, "learn_beta must be 0 or 1");
  if ((cfg->adapt_decay == nullptr) != (cfg->adapt_step == nullptr))
    return fail(nullptr, SNN_ERR_NULL, "adapt_decay and adapt_step must both be given or both be NULL");
  if (cfg->adapt_step)
    for (int i = 0; i < cfg->n_layers - 1; ++i) {
      if (!(cfg->adapt_decay[i] >= 0.f && cfg->adapt_decay[i] <= 1.f)) return fail(nullptr, SNN_ERR_ARG, "adapt_decay[%d] outside [0,1]", i);
      if (!(cfg->adapt_step[i] >= 0.f)) return fail(nullptr, SNN_ERR_ARG, "adapt_step[%d] is negative", i);
      if (cfg->adapt_step[i] > 0.f && cfg->recurrent && cfg->recurrent[i])
        return fail(nullptr, SNN_ERR_UNSUPPORTED, "layer %d is recurrent and adaptive: adaptive thresholds are built for feed-forward layers", i + 1);
    }
  if ((long long)cfg->T * cfg->B > (1ll << 30)) return fail(nullptr, SNN_ERR_ARG, "T*B too large");
  for (int i = 0; i <= cfg->n_layers; ++i)      // byte offsets into one tensor are 31-bit
    if ((long long)cfg->T * cfg->B * (cfg->sizes[i] + 8) * 4 >= (1ll << 31))
      return fail(nullptr, SNN_ERR_ARG, "T*B*sizes[%d] too large: a tensor must stay below 2 GiB", i);
  return SNN_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};
hipError_t static_scratch(void **out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// Contraction splits of the weight-gradient products, which share one launch with `tiles`
// output tiles in total over M rows each.  `weights`: elements of all gradient matrices (a
// split writes that many partial sums); `row_bytes`: operand bytes the products read per row
// of the contraction.  Measured facts behind the rule:
//   * the splits of a tile are dealt round-robin to the 8 XCDs (see gemm_body), so a count
//     that is not a multiple of 8 leaves some XCDs with a split more than others and the
//     launch lasts as long as the fullest (700-512-512-20, T*B = 65536: 21 splits 253 us,
//     24 splits 225 us, 32 splits 180 us);
//   * 512 workgroups run at once (two per compute unit).  Slightly more than that (24 splits
//     x 22 tiles = 528) is the worst case: the stragglers run a whole workgroup's work alone.
//     Either everything fits at once, or there are at least 1.3 rounds of shorter workgroups;
//   * every split writes and the reduction re-reads all partial sums: with large matrices
//     (2048 wide: 56 MB per split) more splits cost more than they gain (64 splits: 10.2 ms
//     against 3.3 ms with 8), and 16 splits never beat 8 at 1024 wide.
//   * the kernel on transposing LDS reads (wgrad_tr.hpp) multiplies as fast with one workgroup per
//     compute unit as with two (its MFMAs are fed by the wavefront's own instruction stream), so for
//     it (`one_per_cu`) half as many splits cover the chip at the same product time and half the
//     partial sums (700-128-128-20, T*B = 32768: 32 splits 19.1 us + 4.4 us for the update against
//     64 splits 20.7 + 6.5);
//   * 2..7 splits would leave whole XCDs without work (a split lives on one XCD): 8 then.
int choose_splits(long long M, int tiles, long long weights, long long row_bytes, long long *per_split, bool one_per_cu) {
  const long long target = 512;                          // workgroups resident at once
  if (tiles < 1) tiles = 1;
  const long long max_by_len = M / 256;                  // at least four 64-row tiles per workgroup
  long long want = target / tiles;
  if (want > max_by_len) want = max_by_len;
  if (want < 1) want = 1;
  if (want > 1 && want < 8 && max_by_len >= 8) want = 8;
  if (want >= 8) {
    want = want / 8 * 8;                                 // all at once, balanced over the XCDs
    // when that leaves more than 15 % of the chip idle: more, shorter workgroups, as long as
    // each keeps 16 tiles of the contraction and the partial sums stay below a quarter of the
    // operand bytes
    const long long more = ((target * 13 / 10 + tiles - 1) / tiles + 7) / 8 * 8;
    if (want * tiles * 100 < target * 85 && M / more >= 1024 && more * weights * 4 * 4 <= M * row_bytes) want = more;
    const long long half = (target / 2 / tiles) / 8 * 8; // one workgroup per compute unit
    if (one_per_cu && half >= 8 && half < want && half * tiles * 100 >= target / 2 * 85) want = half;
  }
  long long per = (long long)rup((size_t)((M + want - 1) / want), 64);
  *per_split = per;
  return (int)((M + per - 1) / per);
}

int wgrad_tiles(int rows, int cols, bool tall) {
  int bn = cols <= 32 ? 32 : (cols <= 64 ? 64 : 128);
  const int bm = tall && cols > 64 ? 256 : 128;
  return ((rows + bm - 1) / bm) * ((cols + bn - 1) / bn);
}

// Rows of C per workgroup for the products over all T*B rows whose output is wider than 64
// columns: the tallest tile that still gives every compute unit a few workgroups.
int pick_rows_per_tile(const snn_ctx *c, long long rows, int cols) {
  const int forced = c->opt[SNN_OPT_TILE_ROWS];
  if (forced == 32 || forced == 64 || forced == 128) return forced;
  const long long col_tiles = (cols + 127) / 128;
  if ((rows + 127) / 128 * col_tiles >= 512) return 128;
  if ((rows + 63) / 64 * col_tiles >= 512) return 64;
  return 32;
}

// Walks the workspace layout; with base == nullptr it only counts.
struct Carver {
  char *base;
  size_t off = 0;
  explicit Carver(char *b) : base(b) {}
  template <typename Tp> Tp *take(size_t n_elems) {
    size_t bytes = rup(n_elems * sizeof(Tp), 256);
    Tp *p = base ? (Tp *)(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

void carve(snn_ctx &c, Carver &cv) {
  const size_t M = (size_t)c.M;
  const int np = c.nplanes;
  // Output tiles of all weight-gradient products (they share one launch).  With many tiles
  // the products are large enough for 256 x 128 tiles, which move 1.7 times fewer operand
  // bytes per flop (measured 2.8 times faster at 1024-wide layers, slower at 128-wide ones).
  auto count_tiles = [&](bool tall) {
    int n = 0;
    for (int l = 0; l < c.L; ++l) {
      n += wgrad_tiles(c.layers[l].K, c.layers[l].N, tall);
      if (c.layers[l].recurrent) n += wgrad_tiles(c.layers[l].N, c.layers[l].N, tall);
    }
    return n;
  };
  c.wg_tall = c.precision != SNN_PREC_FP32 && count_tiles(false) >= 32;
  // (the splits are laid out here, for the kernel that SNN_OPT_WGRAD_TR selects at this point)
  bool wg_tr = c.opt[SNN_OPT_WGRAD_TR] && c.precision != SNN_PREC_FP32;
  {
    bool any_wide = false;
    for (int l = 0; l < c.L; ++l) any_wide = any_wide || c.layers[l].N > 64;
    wg_tr = wg_tr && any_wide;
  }
  const int wg_tiles = count_tiles(c.wg_tall && !wg_tr);
  long long wg_weights = 0, wg_row_bytes = 0;             // what the merged launch writes per split / reads per row
  for (int l = 0; l < c.L; ++l) {
    const Layer &y = c.layers[l];
    wg_weights += (long long)y.K * y.N + (y.recurrent ? (long long)y.N * y.N : 0);
    wg_row_bytes += y.K + 4ll * y.N + (y.recurrent ? y.N : 0);   // spike bytes below, 4-byte current gradients
  }
  for (int l = 0; l < c.L; ++l) {
    Layer &y = c.layers[l];
    const size_t K = y.K, N = y.N;
    y.Wm = cv.take<float>(K * N);
    y.dW = cv.take<float>(K * N);
    y.ldqf = (int)rup(K, 64);
    y.qf_plane = (long long)rup(N, 128) * y.ldqf;
    y.Qf = cv.take<uint16_t>((size_t)np * y.qf_plane);
    if (l > 0) {
      y.ldqb = (int)rup(N, 64);
      y.qb_plane = (long long)rup(K, 128) * y.ldqb;
      y.Qb = cv.take<uint16_t>((size_t)np * y.qb_plane);
    }
    // (layer 1: from the length of the contraction in packed order, T rounded up to whole bytes of
    // eight steps, so that the same splits serve a raster packed along time)
    y.splits_w = choose_splits(l == 0 ? (long long)((c.T + 7) / 8 * 8) * c.B : c.M, wg_tiles, wg_weights, wg_row_bytes, &y.per_w, wg_tr);
    if (y.splits_w > 1) y.part_w = cv.take<float>((size_t)y.splits_w * K * N);
    if (y.recurrent) {
      y.Rm = cv.take<float>(N * N);
      y.dR = cv.take<float>(N * N);
      y.ldqr = (int)rup(N, 64);
      y.qr_plane = (long long)rup(N, 128) * y.ldqr;
      y.QRf = cv.take<uint16_t>((size_t)np * y.qr_plane);
      y.QRb = cv.take<uint16_t>((size_t)np * y.qr_plane);
      y.g[0] = cv.take<float>((size_t)c.B * y.ld);
      y.g[1] = cv.take<float>((size_t)c.B * y.ld);
      if (c.precision != SNN_PREC_FP32 && rlif_persist_fits(c.B, y.ld, y.ldqr, 1 << 30))
        y.rp_space = cv.take<char>(rlif_persist_bytes(c.B, y.ldqr));
      y.splits_r = choose_splits(c.M, wg_tiles, wg_weights, wg_row_bytes, &y.per_r, wg_tr);
      if (y.splits_r > 1) y.part_r = cv.take<float>((size_t)y.splits_r * N * N);
    }
    y.beta_v = cv.take<float>(y.ld);
    y.dbeta = cv.take<float>(y.ld);
    if (c.learn_beta) y.part_b = cv.take<float>((size_t)c.B * y.ld);
    y.I = cv.take<float>(M * y.ld);
    y.V = cv.take<float>(M * y.ld);
    y.dI = cv.take<uint32_t>(M * y.ld);
    if (y.spiking) {
      y.S = cv.take<uint8_t>(M * y.ld);
      y.dS = cv.take<float>(M * y.ld);
    }
    if (y.adaptive) y.A = cv.take<float>(M * y.ld);
  }
  c.ldx = c.sizes[0] % 4 == 0 ? c.sizes[0] : (int)rup(c.sizes[0], 8);
  c.x_padded = c.ldx != c.sizes[0];
  c.x_buf = cv.take<uint8_t>(M * c.ldx);
  c.z = cv.take<float>((size_t)c.B * c.ldC);
  c.dz = cv.take<float>((size_t)c.B * c.ldC);
  c.tstar = cv.take<int>((size_t)c.B * c.ldC);
  c.hand_parts = 1;                                    // column blocks of the widest layer (64 neurons at least each)
  for (const Layer &y : c.layers) c.hand_parts = std::max(c.hand_parts, y.ld / 64);
  c.hand = cv.take<uint32_t>(rup(c.B, 8) * c.hand_parts * (SNN_HAND_BYTES / 4));
  c.loss_b = cv.take<float>((size_t)c.B);
  c.loss = cv.take<float>(64);
  c.err_flag = cv.take<int>(64);
}

void configure(snn_ctx &c, const snn_config *cfg) {
  c.T = cfg->T; c.B = cfg->B; c.L = cfg->n_layers;
  c.M = (long long)c.T * c.B;
  c.sizes.assign(cfg->sizes, cfg->sizes + c.L + 1);
  c.theta = cfg->threshold; c.slope = cfg->slope;
  c.surrogate = cfg->surrogate; c.precision = cfg->precision;
  c.integral = cfg->loss == SNN_LOSS_INTEGRAL;
  c.learn_beta = cfg->learn_beta != 0;
  c.nplanes = c.precision == SNN_PREC_FP32 ? 3 : 1;
  c.hl = c.precision == SNN_PREC_BF16_GEMM;
  c.layers.assign(c.L, Layer());
  for (int l = 0; l < c.L; ++l) {
    Layer &y = c.layers[l];
    y.K = c.sizes[l]; y.N = c.sizes[l + 1];
    y.ld = (int)rup(y.N, 8);
    y.spiking = l < c.L - 1;
    y.recurrent = y.spiking && cfg->recurrent && cfg->recurrent[l];
    y.beta = cfg->beta[l];
    y.adaptive = y.spiking && cfg->adapt_step && cfg->adapt_step[l] > 0.f;
    if (y.adaptive) { y.gamma = cfg->adapt_decay[l]; y.kappa = cfg->adapt_step[l]; }
  }
  c.C = c.sizes[c.L];
  c.ldC = c.layers[c.L - 1].ld;
}

// ------------------------------------------------------------------ profiling brackets
struct Bracket {
  snn_ctx *c;
  bool on;
  Bracket(snn_ctx *ctx, int cls, int layer1) : c(ctx) {
    on = c->prof.cls == cls && (c->prof.layer == 0 || c->prof.layer == layer1);
    if (on) on = c->prof.seen++ % c->prof.every == 0;
    if (on) {
      if (c->prof.used + 2 > c->prof.ev.size()) {
        if (c->prof.ev.size() >= (1u << 16)) { on = false; return; }
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
        c->prof.ev.push_back(a); c->prof.ev.push_back(b);
      }
      (void)hipEventRecord(c->prof.ev[c->prof.used], c->stream);
    }
  }
  ~Bracket() {
    if (on) {
      (void)hipEventRecord(c->prof.ev[c->prof.used + 1], c->stream);
      c->prof.used += 2;
    }
  }
};

// ------------------------------------------------------------------ launches
// Dynamic decompression of a raster packed along time (Section 2.1.4) into the workspace: for the
// launches that have no loader for the packed form (and for shapes the packed loaders do not take).
int prepare_packed_input(snn_ctx *c, const uint8_t *xp) {
  if (!xp) return fail(c, SNN_ERR_NULL, "packed input raster is NULL");
  const long long n = (long long)((c->T + 7) / 8) * c->B * c->sizes[0];
  hipLaunchKernelGGL(unpack_time_bits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, xp, c->x_buf,
                     c->T, c->B, c->sizes[0], c->ldx);
  HIPCHK(c, hipGetLastError());
  c->x_eff = c->x_buf;
  c->x_unpacked = true;
  return SNN_OK;
}

// Before a launch that reads the input raster as bytes: when the last forward pass consumed the
// packed raster directly, unpack it now (a reader of I^1, a single step on imposed inputs).
int ensure_unpacked_input(snn_ctx *c) {
  if (!c->x_direct || c->x_unpacked) return SNN_OK;
  return prepare_packed_input(c, c->x_packed);
}

// The product kernels read spike rows with 4-byte loads.  A raster whose row length is not a
// multiple of 4 is first copied into a zero-padded buffer of the workspace (one extra pass,
// only for such sizes); otherwise it is read in place.
int prepare_input(snn_ctx *c, const uint8_t *x) {
  if (!x) return fail(c, SNN_ERR_NULL, "input raster is NULL");
  c->x_direct = false;
  c->x_packed = nullptr;
  if (c->x_padded) {
    const long long n = c->M * c->ldx;
    hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, x, c->x_buf,
                       c->M, c->sizes[0], c->ldx);
    HIPCHK(c, hipGetLastError());
    c->x_eff = c->x_buf;
  } else {
    if ((uintptr_t)x % 4 != 0) return fail(c, SNN_ERR_ARG, "x_dev must be 4-byte aligned");
    c->x_eff = x;
  }
  return SNN_OK;
}

// Spikes feeding layer index l: the input raster for l == 0, else S of the layer below.
struct SpikeSrc { const uint8_t *p; int ld; int valid; unsigned bytes; };
SpikeSrc spikes_below(snn_ctx *c, int l) {
  if (l == 0) return {c->x_eff, c->ldx, c->ldx, (unsigned)(c->M * c->ldx)};
  return {c->layers[l - 1].S, c->layers[l - 1].ld, c->layers[l - 1].ld, (unsigned)(c->M * c->layers[l - 1].ld)};
}

// A result this large is out of every cache level (L2 8 x 4 MiB, memory-side cache 256 MiB)
// again before the next kernel reads it; stored non-temporally it at least leaves the
// operands of the product that writes it in place.  Smaller results are stored normally: the
// next kernel finds them warm.
// (SNN_OPT_STREAM_MIN_MB moves the limit; the tests set it to 0 to run these paths on small shapes.)
static bool streams_past_cache(const snn_ctx *c, size_t bytes) {
  return bytes >= ((size_t)c->opt[SNN_OPT_STREAM_MIN_MB] << 20);
}

static bool stream_gemm(const snn_ctx *c) { return c->opt[SNN_OPT_STREAM_GEMM] != 0; }

// I^l = S^{l-1} W^l over all T*B rows at once.
int launch_current_gemm(snn_ctx *c, int l) {
  Layer &y = c->layers[l];
  if (l == 0) { int rc = ensure_unpacked_input(c); if (rc) return rc; }
  SpikeSrc s = spikes_below(c, l);
  if (!s.p) return fail(c, SNN_ERR_NULL, "input raster is NULL");
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.P = s.p; a.ldp = s.ld; a.kc = s.valid; a.p_bytes = s.bytes;
  a.Q = y.Qf; a.ldq = y.ldqf; a.q_plane_stride = y.qf_plane; a.q_bytes = (unsigned)(c->nplanes * y.qf_plane * 2);
  a.C = y.I; a.ldc = y.ld; a.rows = (int)c->M; a.cols = y.N;
  a.kc_per_split = (int)rup(a.kc, 64);
  a.nt_store = streams_past_cache(c, c->M * y.ld * 4);
  Bracket br(c, SNN_K_CURRENT_GEMM, l + 1);
  hipError_t e;
  const int bm = pick_rows_per_tile(c, c->M, y.N);
  // The streamed kernel addresses both P and C with 32-bit byte offsets.
  const bool streamed = a.nt_store && stream_gemm(c) && c->M * y.ld * 4 < ((size_t)1 << 31) && (size_t)c->M * s.ld < ((size_t)1 << 31);
  if (c->precision == SNN_PREC_FP32) {
    if (y.N <= 32) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 4, 1, 1, 1, 3, 1>(a, 1, c->stream);
    else if (y.N <= 64) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 2, 1, 3, 1>(a, 1, c->stream);
    else if (bm == 128) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 2, 2, 3, 1>(a, 1, c->stream);
    else if (bm == 64) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 1, 2, 3, 1>(a, 1, c->stream);
    else e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 1, 4, 1, 1, 3, 1>(a, 1, c->stream);
  } else {
    if (y.N <= 32) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 4, 1, 1, 1, 1, 1>(a, 1, c->stream);
    else if (y.N <= 64) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 2, 1, 1, 1>(a, 1, c->stream);
    else if (bm == 128 && y.N >= 256 && streamed) e = spike_gemm_launch<2, 2, 2, 4>(a, c->stream);
    else if (bm == 128 && streamed) e = spike_gemm_launch<2, 2, 2, 2>(a, c->stream);
    else if (bm == 128 && y.N >= 256) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 2, 4, 1, 1>(a, 1, c->stream);
    else if (bm == 128) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 2, 2, 1, 1>(a, 1, c->stream);
    else if (bm == 64) e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 2, 2, 1, 2, 1, 1>(a, 1, c->stream);
    else e = gemm_launch<P_U8, Q_BF16, EPI_STORE, 1, 4, 1, 1, 1, 1>(a, 1, c->stream);
  }
  HIPCHK(c, e);
  y.i_ready = true;
  return SNN_OK;
}

// dS^{l-1} = dI^l W^l^T  (l >= 1).
int launch_input_grad(snn_ctx *c, int l) {
  Layer &y = c->layers[l];
  Layer &below = c->layers[l - 1];
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.P = y.dI; a.ldp = y.ld; a.kc = y.ld; a.p_bytes = (unsigned)(c->M * y.ld * 4);
  a.Q = y.Qb; a.ldq = y.ldqb; a.q_plane_stride = y.qb_plane; a.q_bytes = (unsigned)(c->nplanes * y.qb_plane * 2);
  a.C = below.dS; a.ldc = below.ld; a.rows = (int)c->M; a.cols = y.K;
  a.kc_per_split = (int)rup(a.kc, 64);
  a.nt_store = streams_past_cache(c, c->M * below.ld * 4);
  Bracket br(c, SNN_K_INPUT_GRAD, l + 1);
  hipError_t e;
  const int bm = pick_rows_per_tile(c, c->M, y.K);
  if (c->precision == SNN_PREC_FP32) {
    if (y.K <= 32) e = gemm_launch<P_F32S, Q_BF16, EPI_STORE, 4, 1, 1, 1, 3, 1>(a, 1, c->stream);
    else e = gemm_launch<P_F32S, Q_BF16, EPI_STORE, 2, 2, 1, 1, 3, 1>(a, 1, c->stream);
  } else {
    if (y.K <= 32) e = gemm_launch<P_HL, Q_BF16, EPI_STORE, 4, 1, 1, 1, 1, 1>(a, 1, c->stream);
    else if (bm == 128) e = gemm_launch<P_HL, Q_BF16, EPI_STORE, 2, 2, 2, 2, 1, 1>(a, 1, c->stream);
    else if (bm == 64) e = gemm_launch<P_HL, Q_BF16, EPI_STORE, 2, 2, 1, 2, 1, 1>(a, 1, c->stream);
    else e = gemm_launch<P_HL, Q_BF16, EPI_STORE, 1, 4, 1, 1, 1, 1>(a, 1, c->stream);
  }
  HIPCHK(c, e);
  return SNN_OK;
}

// part[split][rows x cols] (or out directly when there is one split) = Sp^T G over one
// slice of the T*B rows per split.
// Transposed products S^T G (weight gradients), gathered by tile shape: the products of all
// layers are independent of each other and of the rest of the backward pass once their
// operands exist, so they are launched together after the last reverse scan.
struct WgradJobs {
  GemmJobs narrow, mid, wide;        // cols <= 32, <= 64, wider
};

// The wide products on rounded weights go through the kernel built on transposing LDS reads
// (SNN_OPT_WGRAD_TR, 128 x 128 tiles), else through the general one (256 x 128 tiles when there are many).
static bool wgrad_tr(const snn_ctx *c) { return c->opt[SNN_OPT_WGRAD_TR] && c->precision != SNN_PREC_FP32; }
static bool wgrad_tall(const snn_ctx *c) { return c->wg_tall && !wgrad_tr(c); }

int flush_tn(snn_ctx *c, WgradJobs &w, int which) {
  hipError_t e = hipSuccess;
  const bool f32 = c->precision == SNN_PREC_FP32;
  if (which == 0 && w.narrow.njobs) {
    e = f32 ? gemm_jobs_launch<P_T_U8, Q_T_F32S, EPI_STORE, 4, 1, 1, 1, 3, 1>(w.narrow, c->stream)
            : gemm_jobs_launch<P_T_U8, Q_T_HL, EPI_STORE, 4, 1, 1, 1, 2, 1>(w.narrow, c->stream);
    memset(&w.narrow, 0, sizeof w.narrow);
  } else if (which == 1 && w.mid.njobs) {
    e = f32 ? gemm_jobs_launch<P_T_U8, Q_T_F32S, EPI_STORE, 2, 2, 2, 1, 3, 1>(w.mid, c->stream)
            : gemm_jobs_launch<P_T_U8, Q_T_HL, EPI_STORE, 2, 2, 2, 1, 2, 1>(w.mid, c->stream);
    memset(&w.mid, 0, sizeof w.mid);
  } else if (which == 2 && w.wide.njobs) {
    e = f32 ? gemm_jobs_launch<P_T_U8, Q_T_F32S, EPI_STORE, 2, 2, 2, 2, 3, 1>(w.wide, c->stream)
            : wgrad_tr(c) ? wgrad_tr_jobs_launch(w.wide, c->stream)
            : c->wg_tall ? gemm_jobs_launch<P_T_U8, Q_T_HL, EPI_STORE, 2, 2, 4, 2, 2, 1>(w.wide, c->stream)
                           : gemm_jobs_launch<P_T_U8, Q_T_HL, EPI_STORE, 2, 2, 2, 2, 2, 1>(w.wide, c->stream);
    memset(&w.wide, 0, sizeof w.wide);
  }
  HIPCHK(c, e);
  return SNN_OK;
}

int queue_tn(snn_ctx *c, WgradJobs &w, SpikeSrc s, int rows, const void *G, int ldg, int cols, float *out,
             float *part, int splits, long long per, bool packed = false) {
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.P = s.p; a.ldp = s.ld; a.p_ivalid = s.valid; a.p_bytes = s.bytes;
  a.Q = G; a.ldq = ldg; a.q_bytes = (unsigned)(c->M * ldg * 4);
  a.rows = rows; a.cols = cols; a.ldc = cols; a.kc = (int)c->M;
  if (packed) {                    // P packed along time: the contraction in packed order, whole bytes of eight steps
    a.packed = 1; a.pk_T = c->T; a.pk_B = c->B;
    a.kc = (c->T + 7) / 8 * 8 * c->B;
  }
  a.kc_per_split = (int)per;
  a.c_split_stride = (long long)rows * cols;
  a.C = splits > 1 ? part : out;
  const int which = cols <= 32 ? 0 : cols <= 64 ? 1 : 2;
  GemmJobs &list = which == 0 ? w.narrow : which == 1 ? w.mid : w.wide;
  if (list.njobs == SNN_GEMM_MAX_JOBS) {
    int rc = flush_tn(c, w, which);
    if (rc) return rc;
  }
  if (which == 0) gemm_jobs_add<4, 1, 1, 1>(list, a, splits);
  else if (which == 1) gemm_jobs_add<2, 2, 2, 1>(list, a, splits);
  else if (wgrad_tall(c)) gemm_jobs_add<2, 2, 4, 2>(list, a, splits);
  else gemm_jobs_add<2, 2, 2, 2>(list, a, splits);
  return SNN_OK;
}

static_assert(SNN_MAX_REDUCE_JOBS >= 3 * SNN_MAX_LAYERS, "dW, dR and dbeta of every layer");
static_assert(SNN_MAX_JOBS >= 2 * SNN_MAX_LAYERS, "W and R of every layer");
bool add_reduce_job(ReduceJobs &jobs, const float *part, float *out, int splits, long long n, bool always = false) {
  if (splits <= 1 && !always) return true;  // a single split was written straight to `out`
  if (jobs.njobs >= SNN_MAX_REDUCE_JOBS) return false;
  const int j = jobs.njobs++;
  jobs.part[j] = part; jobs.out[j] = out; jobs.splits[j] = splits; jobs.n[j] = n;
  jobs.first_block[j + 1] = jobs.first_block[j] + (int)((n + 255) / 256);
  return true;
}

// Sums the split partial products; with_loss adds the workgroup that takes the mean loss.
int launch_reduce(snn_ctx *c, const ReduceJobs &jobs, bool with_loss) {
  const int blocks = jobs.first_block[jobs.njobs] + (with_loss ? 1 : 0);
  if (blocks == 0) return SNN_OK;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, c->stream, jobs,
                     with_loss ? c->loss_b : nullptr, c->loss, c->B);
  HIPCHK(c, hipGetLastError());
  if (with_loss) c->loss_ready = true;
  return SNN_OK;
}

int ensure_loss(snn_ctx *c) {
  if (c->loss_ready) return SNN_OK;
  hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(256), 0, c->stream, c->loss_b, c->loss, c->B);
  HIPCHK(c, hipGetLastError());
  c->loss_ready = true;
  return SNN_OK;
}

// dW^l = S^{l-1}^T dI^l and, for a recurrent layer, dR^l = S^l^T dI^l: the split products
// are queued on `w`, their partial sums on `jobs` (one reduction launch for all layers).
int queue_weight_grad(snn_ctx *c, int l, WgradJobs &w, ReduceJobs &jobs) {
  Layer &y = c->layers[l];
  // Layer 1 after a forward pass on the packed raster: the product reads the bits itself when the
  // batch is a multiple of 8 (its contraction tiles are eight samples wide); else unpack first.
  const bool packed = l == 0 && c->x_direct && !c->x_unpacked && c->B % 8 == 0;
  if (l == 0 && !packed) { int rc = ensure_unpacked_input(c); if (rc) return rc; }
  SpikeSrc s = spikes_below(c, l);
  if (packed) s = {c->x_packed, c->sizes[0], c->sizes[0], (unsigned)((long long)((c->T + 7) / 8) * c->B * c->sizes[0])};
  if (!s.p) return fail(c, SNN_ERR_NULL, "input raster is NULL");
  int rc = queue_tn(c, w, s, y.K, y.dI, y.ld, y.N, y.dW, y.part_w, y.splits_w, y.per_w, packed);
  if (rc) return rc;
  bool ok = add_reduce_job(jobs, y.part_w, y.dW, y.splits_w, (long long)y.K * y.N);
  if (y.recurrent) {
    SpikeSrc own = {y.S, y.ld, y.ld, (unsigned)(c->M * y.ld)};
    rc = queue_tn(c, w, own, y.N, y.dI, y.ld, y.N, y.dR, y.part_r, y.splits_r, y.per_r);
    ok = ok && add_reduce_job(jobs, y.part_r, y.dR, y.splits_r, (long long)y.N * y.N);
  }
  if (!ok) return fail(c, SNN_ERR_UNSUPPORTED, "more than %d gradient reductions in one backward pass", SNN_MAX_REDUCE_JOBS);
  return rc;
}

// Launches what was queued (largest tiles first) and the reduction of the partial sums.
int launch_weight_grads(snn_ctx *c, WgradJobs &w, const ReduceJobs &jobs, bool with_loss, bool defer = false) {
  int rc;
  {
  Bracket br(c, SNN_K_WEIGHT_GRAD, 0);
  // A narrow product (the readout's) is small; when a launch with wide tiles exists it rides
  // along there (its tile count is the same, the unused columns load zeros) rather than
  // paying for a launch of its own.
  for (GemmJobs *from : {&w.narrow, &w.mid})
    while (from->njobs && w.wide.njobs && w.wide.njobs < SNN_GEMM_MAX_JOBS) {
      const GemmArgs a = from->job[--from->njobs];
      if (wgrad_tall(c)) gemm_jobs_add<2, 2, 4, 2>(w.wide, a, a.splits);
      else gemm_jobs_add<2, 2, 2, 2>(w.wide, a, a.splits);
    }
  for (int which = 2; which >= 0; --which)
    if ((rc = flush_tn(c, w, which))) return rc;
  }
  if (defer) {                     // snn_sgd_step (or the first reader of a gradient) adds the partial sums
    c->pending = jobs;
    c->reduce_pending = true;
    return SNN_OK;
  }
  c->reduce_pending = false;
  Bracket br(c, SNN_K_GRAD_REDUCE, 0);
  return launch_reduce(c, jobs, with_loss);
}

// Adds partial sums that snn_backward left for snn_sgd_step, for a caller that wants the
// gradients (or anything else) first.
int flush_reduce(snn_ctx *c) {
  if (!c->reduce_pending) return SNN_OK;
  c->reduce_pending = false;
  Bracket br(c, SNN_K_GRAD_REDUCE, 0);
  return launch_reduce(c, c->pending, !c->loss_ready);
}

// Threads per workgroup of the one-thread-per-chain scans: single wavefronts while that is
// what it takes to give each of the 256 compute units (8 XCDs x 32) something to do.
int scan_block(long long threads) { return threads >= 256 * 1024 ? 256 : 64; }

template <int VEC, int U>
hipError_t lif_fwd_launch(snn_ctx *c, Layer &y) {
  const int stride = c->B * y.ld;               // T * stride * 4 < 2 GiB was checked at init
  const int threads = stride / VEC;
  const int bs = scan_block(threads);
  const dim3 grid((unsigned)((threads + bs - 1) / bs)), block(bs);
  const bool nt = streams_past_cache(c, c->M * y.ld * 4);
#define SNN_FWD(POL_, AD_)                                                                                       \
  hipLaunchKernelGGL((lif_forward_kernel<VEC, U, POL_, AD_>), grid, block, 0, c->stream, y.I, y.V, y.S, c->T, stride, \
                     y.beta_v, y.ld, c->theta, y.A, y.gamma, y.kappa)
  if (y.adaptive) { if (nt) SNN_FWD(NT, true); else SNN_FWD(0, true); }
  else { if (nt) SNN_FWD(NT, false); else SNN_FWD(0, false); }
#undef SNN_FWD
  return hipGetLastError();
}

int launch_lif_forward(snn_ctx *c, int l) {
  Layer &y = c->layers[l];
  if (y.recurrent) {
    Bracket br(c, SNN_K_RLIF_FORWARD, l + 1);
    // a wide layer on rounded weights whose grid fits the compute units at one workgroup each: the whole
    // time loop in one launch (SNN_OPT_RLIF_PERSIST), else a launch per step
    if (c->opt[SNN_OPT_RLIF_PERSIST] && y.rp_space && c->T >= 2 && rlif_persist_fits(c->B, y.ld, y.ldqr, c->cus)) {
      HIPCHK(c, rlif_persist_forward(c->stream, c->T, c->B, y.ld, y.I, y.V, y.S, y.QRf, y.ldqr, y.beta_v, c->theta,
                                     y.rp_space, c->err_flag, 1 << c->opt[SNN_OPT_WAIT_LIMIT_LOG2], c->opt[SNN_OPT_WAIT_FAULT] != 0));
      return SNN_OK;
    }
    HIPCHK(c, rlif_forward(c->stream, c->precision == SNN_PREC_FP32, c->T, c->B, y.N, y.ld, y.I, y.V, y.S, y.QRf,
                           y.ldqr, y.qr_plane, y.beta_v, c->theta));
    return SNN_OK;
  }
  Bracket br(c, SNN_K_LIF_FORWARD, l + 1);
  const long long chains = (long long)c->B * y.ld;
  hipError_t e;
  if (chains >= (1 << 19)) e = lif_fwd_launch<4, 8>(c, y);
  else if (chains >= (1 << 17)) e = lif_fwd_launch<2, 16>(c, y);
  else e = lif_fwd_launch<1, 16>(c, y);
  HIPCHK(c, e);
  return SNN_OK;
}

template <int VEC, int U, bool HL>
hipError_t lif_rev_launch2(snn_ctx *c, Layer &y) {
  const int stride = c->B * y.ld;
  const int threads = stride / VEC;
  const int bs = scan_block(threads);
  dim3 grid((unsigned)((threads + bs - 1) / bs)), block(bs);
  const bool nt = streams_past_cache(c, c->M * y.ld * 4);
#define SNN_REV2(SU, POL_, AD_)                                                                                  \
  hipLaunchKernelGGL((lif_reverse_kernel<VEC, U, SU, HL, POL_, AD_>), grid, block, 0, c->stream, y.dS, y.V, y.dI, c->T, \
                     stride, y.beta_v, y.ld, c->theta, c->slope, y.part_b, y.A, y.gamma, y.kappa)
#define SNN_REV(SU)                                                                                              \
  do {                                                                                                           \
    if (y.adaptive) { if (nt) SNN_REV2(SU, NT, true); else SNN_REV2(SU, 0, true); }                              \
    else { if (nt) SNN_REV2(SU, NT, false); else SNN_REV2(SU, 0, false); }                                       \
  } while (0)
  switch (c->surrogate) {
    case 0: SNN_REV(0); break;
    case 1: SNN_REV(1); break;
    case 2: SNN_REV(2); break;
    case 3: SNN_REV(3); break;
    case 4: SNN_REV(4); break;
    default: SNN_REV(5); break;
  }
#undef SNN_REV
#undef SNN_REV2
  return hipGetLastError();
}
template <int VEC, int U>
hipError_t lif_rev_launch(snn_ctx *c, Layer &y) {
  return c->hl ? lif_rev_launch2<VEC, U, true>(c, y) : lif_rev_launch2<VEC, U, false>(c, y);
}

int launch_lif_reverse(snn_ctx *c, int l) {
  Layer &y = c->layers[l];
  if (y.recurrent) {
    Bracket br(c, SNN_K_RLIF_REVERSE, l + 1);
    HIPCHK(c, rlif_reverse(c->stream, c->precision == SNN_PREC_FP32, c->T, c->B, y.N, y.ld, y.dS, y.V, y.dI,
                           y.g[0], y.g[1], y.QRb, y.ldqr, y.qr_plane, y.beta_v, c->theta, c->surrogate, c->slope,
                           y.part_b));
    return SNN_OK;
  }
  Bracket br(c, SNN_K_LIF_REVERSE, l + 1);
  const long long chains = (long long)c->B * y.ld;
  hipError_t e;
  if (chains >= (1 << 19)) e = lif_rev_launch<4, 4>(c, y);
  else if (chains >= (1 << 17)) e = lif_rev_launch<2, 8>(c, y);
  else e = lif_rev_launch<1, 16>(c, y);
  HIPCHK(c, e);
  return SNN_OK;
}

// A spiking layer can take dS = dX W^T from the current gradients dX of the layer above inside
// its reverse scan (lif_reverse_top_kernel) when it is feed-forward, its rows hold whole
// wavefronts (ld a multiple of 64), the layer above has at most 128 padded columns (the
// readout, or a narrow spiking layer) and the products run on rounded weights.  (One chain per
// lane also at large widths: at 1024 neurons below the readout the fused scan takes 216 us
// where the four-chains-per-lane scan plus the readout's input-gradient launch took 290 + 100.)
int columns_above(const snn_ctx *c, int l) { return l + 1 == c->L - 1 ? c->ldC : c->layers[l + 1].ld; }
// Below a WIDER layer (more than 128 columns) the whole reverse layer can run as one launch whose
// dS product walks the long contraction on the streamed pipeline (lif_layer_reverse_kernel, WIDE):
// layers that are a multiple of 128 wide, as many samples as the one-launch layers ask for.
// Only on request (SNN_OPT_LAYER_REVERSE = 2): measured, it is slower than the input-gradient
// product followed by the scan at every width tried (700-512-512-20, 256 steps, 256 samples: 195 us
// against 84 + 69; 700-1024-1024-20, 256 steps, 512 samples: 1421 us against 526 + 270).  A
// workgroup walks one sample through time, so the 64 rows of a block lie B x columns x 4 bytes
// apart (2 MiB at the second shape), every stage waits out a full memory latency with three stages
// (48 KiB) in flight per compute unit, and the weights of its 128 neurons (256 KiB) pass through
// the compute unit again for every 64 steps.
bool reverse_wide(const snn_ctx *c, int l) {
  if (c->opt[SNN_OPT_LAYER_REVERSE] != 2 || l < 0 || l > c->L - 2) return false;
  const Layer &y = c->layers[l];
  const int min_b = c->opt[SNN_OPT_LAYER_MIN_BATCH] > 0 ? c->opt[SNN_OPT_LAYER_MIN_BATCH] : c->T <= 256 ? 1 : 64;
  return c->hl && y.spiking && !y.recurrent && !y.adaptive && y.ld % 128 == 0 && columns_above(c, l) > 128 && c->B >= min_b;
}
bool reverse_fusable(const snn_ctx *c, int l) {
  if (l < 0 || l > c->L - 2) return false;
  if (reverse_wide(c, l)) return true;
  if (!c->opt[SNN_OPT_TOP_SCANS]) return false;
  const Layer &y = c->layers[l];
  return c->hl && y.spiking && !y.recurrent && !y.adaptive && y.ld % 64 == 0 && columns_above(c, l) <= 128;
}

// Forward counterpart: the last spiking layer's scan also forms the readout's currents
// (lif_forward_top_kernel), one workgroup per sample.
bool top_forward_fusable(const snn_ctx *c) {
  if (c->L < 2 || !reverse_fusable(c, c->L - 2)) return false;
  const int ld = c->layers[c->L - 2].ld;
  return c->nplanes == 1 && c->ldC <= 32 && (ld == 64 || ld == 128 || ld == 256);
}

int launch_lif_forward_top(snn_ctx *c) {
  const int l = c->L - 2;
  Layer &y = c->layers[l];
  Layer &ro = c->layers[c->L - 1];
  Bracket br(c, SNN_K_LIF_FORWARD, l + 1);
  const int stride = c->B * y.ld;
  const int q_rows = (int)(ro.qf_plane / ro.ldqf);
  const bool nt = streams_past_cache(c, c->M * y.ld * 4);
#define SNN_FWDT(NW)                                                                                              \
  do {                                                                                                            \
    if (nt)                                                                                                       \
      hipLaunchKernelGGL((lif_forward_top_kernel<NW, NT>), dim3(c->B), dim3(64 * NW), 0, c->stream, y.I, y.V, y.S, ro.I, \
                         c->ldC, ro.Qf, ro.ldqf, q_rows, c->T, c->B, stride, y.beta_v, c->theta);                  \
    else                                                                                                          \
      hipLaunchKernelGGL((lif_forward_top_kernel<NW, 0>), dim3(c->B), dim3(64 * NW), 0, c->stream, y.I, y.V, y.S, ro.I,  \
                         c->ldC, ro.Qf, ro.ldqf, q_rows, c->T, c->B, stride, y.beta_v, c->theta);                  \
  } while (0)
  if (y.ld == 64) SNN_FWDT(1);
  else if (y.ld == 128) SNN_FWDT(2);
  else SNN_FWDT(4);
#undef SNN_FWDT
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

// The same reverse pass as one workgroup per sample and 64 neurons on LDS
// (lif_layer_reverse_kernel): layers of 64 to 256 neurons (wider, the scan with a wavefront per
// 64 chains is faster: 121 against 129 us at 512 neurons, 466 against 492 at 1024), 32-bit byte
// offsets.  SNN_OPT_LAYER_REVERSE = 0 switches it off; SNN_OPT_LAYER_MIN_BATCH as for the forward pass.
int layer_min_batch(const snn_ctx *c) {
  return c->opt[SNN_OPT_LAYER_MIN_BATCH] > 0 ? c->opt[SNN_OPT_LAYER_MIN_BATCH] : c->T <= 256 ? 1 : 64;
}
bool layer_reverse_whole(snn_ctx *c, int l) {
  if (!c->opt[SNN_OPT_LAYER_REVERSE]) return false;
  const Layer &y = c->layers[l];
  const int min_b = layer_min_batch(c);
  return reverse_fusable(c, l) && !reverse_wide(c, l) && y.ld <= 256 && c->B >= min_b &&
         (size_t)c->M * y.ld * 4 < ((size_t)1 << 31) && (size_t)c->M * columns_above(c, l) * 4 < ((size_t)1 << 31);
}

int launch_layer_reverse(snn_ctx *c, int l) {
  Layer &y = c->layers[l];
  Layer &up = c->layers[l + 1];
  LayerReverseArgs a;
  memset(&a, 0, sizeof a);
  a.dX = up.dI; a.ldc = columns_above(c, l);
  a.Wq = up.Qb; a.ldq = up.ldqb; a.wq_bytes = (unsigned)(up.qb_plane * 2);
  a.V = y.V; a.dI = y.dI; a.beta_v = y.beta_v; a.theta = c->theta; a.slope = c->slope; a.db_part = y.part_b;
  a.T = c->T; a.B = c->B; a.ld = y.ld;
  a.nt_store = streams_past_cache(c, c->M * y.ld * 4);
  Bracket br(c, SNN_K_LIF_REVERSE, l + 1);
  // 64 neurons per workgroup (two or three workgroups share a compute unit and overlap each
  // other's phases): 99.8 us per step at 700-128-128-20 against 104.8 with 128 neurons.
  const dim3 grid((unsigned)(rup(c->B, 8) * (y.ld / 64))), block(256);
#define SNN_LREV(SU)                                                                                             \
  do {                                                                                                           \
    if (a.ldc <= 32) hipLaunchKernelGGL((lif_layer_reverse_kernel<1, SU, 64>), grid, block, 0, c->stream, a);    \
    else if (a.ldc <= 64) hipLaunchKernelGGL((lif_layer_reverse_kernel<2, SU, 64>), grid, block, 0, c->stream, a); \
    else hipLaunchKernelGGL((lif_layer_reverse_kernel<4, SU, 64>), grid, block, 0, c->stream, a);                \
  } while (0)
  switch (c->surrogate) {
    case 0: SNN_LREV(0); break;
    case 1: SNN_LREV(1); break;
    case 2: SNN_LREV(2); break;
    case 3: SNN_LREV(3); break;
    case 4: SNN_LREV(4); break;
    default: SNN_LREV(5); break;
  }
#undef SNN_LREV
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

int launch_layer_reverse_wide(snn_ctx *c, int l) {
  Layer &y = c->layers[l];
  Layer &up = c->layers[l + 1];
  LayerReverseArgs a;
  memset(&a, 0, sizeof a);
  a.dX = up.dI; a.ldc = columns_above(c, l);
  a.Wq = up.Qb; a.ldq = up.ldqb; a.wq_bytes = (unsigned)(up.qb_plane * 2);
  a.V = y.V; a.dI = y.dI; a.beta_v = y.beta_v; a.theta = c->theta; a.slope = c->slope; a.db_part = y.part_b;
  a.T = c->T; a.B = c->B; a.ld = y.ld;
  a.nt_store = streams_past_cache(c, c->M * y.ld * 4);
  Bracket br(c, SNN_K_LIF_REVERSE, l + 1);
  const dim3 grid((unsigned)(rup(c->B, 8) * (y.ld / 128))), block(256);
  switch (c->surrogate) {
    case 0: hipLaunchKernelGGL((lif_layer_reverse_kernel<1, 0, 128, true>), grid, block, 0, c->stream, a); break;
    case 1: hipLaunchKernelGGL((lif_layer_reverse_kernel<1, 1, 128, true>), grid, block, 0, c->stream, a); break;
    case 2: hipLaunchKernelGGL((lif_layer_reverse_kernel<1, 2, 128, true>), grid, block, 0, c->stream, a); break;
    case 3: hipLaunchKernelGGL((lif_layer_reverse_kernel<1, 3, 128, true>), grid, block, 0, c->stream, a); break;
    case 4: hipLaunchKernelGGL((lif_layer_reverse_kernel<1, 4, 128, true>), grid, block, 0, c->stream, a); break;
    default: hipLaunchKernelGGL((lif_layer_reverse_kernel<1, 5, 128, true>), grid, block, 0, c->stream, a); break;
  }
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

int launch_lif_reverse_fused(snn_ctx *c, int l) {
  if (reverse_wide(c, l)) return launch_layer_reverse_wide(c, l);
  if (layer_reverse_whole(c, l)) return launch_layer_reverse(c, l);
  Layer &y = c->layers[l];
  Layer &up = c->layers[l + 1];
  Bracket br(c, SNN_K_LIF_REVERSE, l + 1);
  const int stride = c->B * y.ld, ldc = columns_above(c, l);
  const int wpg = (y.ld / 64) % 4 == 0 ? 4 : (y.ld / 64) % 2 == 0 ? 2 : 1;   // wavefronts per workgroup: one sample's
  const dim3 grid((unsigned)(stride / 64 / wpg)), block(64 * wpg);
  const bool nt = streams_past_cache(c, c->M * y.ld * 4);
#define SNN_REVT2(KS, SU)                                                                                        \
  do {                                                                                                           \
    if (nt)                                                                                                      \
      hipLaunchKernelGGL((lif_reverse_top_kernel<KS, SU, NT>), grid, block, 0, c->stream, up.dI, ldc, up.Qb, up.ldqb, \
                         y.V, y.dI, c->T, c->B, stride, y.beta_v, y.ld, c->theta, c->slope, y.part_b);           \
    else                                                                                                         \
      hipLaunchKernelGGL((lif_reverse_top_kernel<KS, SU, 0>), grid, block, 0, c->stream, up.dI, ldc, up.Qb, up.ldqb,  \
                         y.V, y.dI, c->T, c->B, stride, y.beta_v, y.ld, c->theta, c->slope, y.part_b);           \
  } while (0)
#define SNN_REVT(SU)                                                                                             \
  do {                                                                                                           \
    if (ldc <= 32) SNN_REVT2(1, SU); else if (ldc <= 64) SNN_REVT2(2, SU);                                       \
    else if (ldc <= 96) SNN_REVT2(3, SU); else SNN_REVT2(4, SU);                                                 \
  } while (0)
  switch (c->surrogate) {
    case 0: SNN_REVT(0); break;
    case 1: SNN_REVT(1); break;
    case 2: SNN_REVT(2); break;
    case 3: SNN_REVT(3); break;
    case 4: SNN_REVT(4); break;
    default: SNN_REVT(5); break;
  }
#undef SNN_REVT
#undef SNN_REVT2
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

// A feed-forward spiking layer of up to 1024 (padded) neurons, a multiple of 64, on rounded
// weights runs as ONE launch, product and scan (lif_layer_forward_kernel): I is not stored.
// A workgroup owns a sample and 64 or 128 neurons; 32-bit
// byte offsets into the spikes below and V; a threshold the scan's compare-free spike
// decision is exact for.
// Width limit (SNN_OPT_LAYER_MAX_NEURONS): the parts of a sample each pass its spike rows below
// through their CU, which the I round trip saved outweighs up to 1024 neurons (product + scan
// 228 -> 169 us at 700-512-512-20, 982 -> 781 us at 700-1024-1024-20, 256 steps) and no longer
// at 2048 (1433 -> 1455 us, 512 steps, 128 samples); the same limit holds for the fan-in.
// SNN_OPT_LAYER_FORWARD: 0 never, 1 all but the last spiking layer, 2 every such layer, 3 the last
// one also forms the readout's currents when it has exactly 128 padded neurons, 4 (default) and
// runs the readout scan, the loss and the readout's current gradients;
// SNN_OPT_LAYER_MIN_BATCH: samples from which it is used (default: any number up to 256 steps, 64
// for longer rasters: at the headline widths it wins from 4 samples on, having fewer launches,
// but a workgroup walks its sample's blocks of 128 steps serially); SNN_OPT_LAYER_NEURONS: 64 or
// 128 neurons per workgroup.
int layer_fuse_mode(const snn_ctx *c) { return c->opt[SNN_OPT_LAYER_FORWARD]; }
static int layer_max_neurons(const snn_ctx *c) { return c->opt[SNN_OPT_LAYER_MAX_NEURONS]; }
bool layer_forward_fusable(snn_ctx *c, int l) {
  if (l < 0 || l > c->L - 2) return false;
  const Layer &y = c->layers[l];
  const int min_b = layer_min_batch(c);                  // a workgroup walks a sample's blocks of 128 steps one after the other
  const SpikeSrc s = spikes_below(c, l);
  return c->nplanes == 1 && y.spiking && !y.recurrent && !y.adaptive && y.ld % 64 == 0 && y.ld <= layer_max_neurons(c) && c->B >= min_b &&
         s.ld % 4 == 0 && s.ld <= layer_max_neurons(c) && (size_t)c->M * s.ld < ((size_t)1 << 31) && (size_t)c->M * y.ld * 4 < ((size_t)1 << 31) &&
         y.qf_plane >= (long long)y.ld * y.ldqf && c->theta >= 0x1p-60f && c->theta <= 0x1p26f;
}

// What the launch of the last spiking layer takes over from the readout: 0 nothing, 1 its
// currents J, 2 also the LI scan, the loss and dJ (what readout_loss_kernel does).
int layer_forward_takes_readout(snn_ctx *c) {
  const Layer &ro = c->layers[c->L - 1];
  const int mode = layer_fuse_mode(c);
  const bool ok = c->L >= 2 && mode >= 3 && layer_forward_fusable(c, c->L - 2) && c->layers[c->L - 2].ld == 128 &&
                  c->opt[SNN_OPT_LAYER_NEURONS] == 128 && c->ldC <= 32 && ro.qf_plane >= 32ll * ro.ldqf && ro.ldqf >= 128;
  return !ok ? 0 : mode >= 4 && c->hl ? 2 : 1;
}

// Layers l .. l + nl - 1 in one launch (nl = 2: both of exactly 128 padded neurons, a workgroup
// takes its sample through both); with_readout refers to the last of them.
int launch_layer_forward(snn_ctx *c, int l, int nl, int with_readout, const int32_t *labels) {
  Layer &y = c->layers[l];
  LayerForwardArgs a;
  memset(&a, 0, sizeof a);
  const bool packed = l == 0 && c->x_direct;           // the bottom layer reads the raster packed along time
  for (int i = 0; i < nl; ++i) {
    Layer &yi = c->layers[l + i];
    SpikeSrc s = spikes_below(c, l + i);
    if (packed && i == 0) s = {c->x_packed, c->sizes[0], c->sizes[0], (unsigned)((long long)((c->T + 7) / 8) * c->B * c->sizes[0])};
    if (!s.p) return fail(c, SNN_ERR_NULL, "input raster is NULL");
    LayerForwardOp &op = a.op[i];
    op.P = s.p; op.ldp = s.ld; op.kc = s.valid; op.p_bytes = s.bytes;
    op.Q = yi.Qf; op.ldq = yi.ldqf; op.q_bytes = (unsigned)(yi.qf_plane * 2);
    op.V = yi.V; op.S = yi.S; op.beta_v = yi.beta_v;
    yi.i_ready = false;
  }
  a.theta = c->theta;
  a.T = c->T; a.B = c->B; a.ld = y.ld;
  a.nt_store = streams_past_cache(c, c->M * y.ld * 4);
  a.err = c->err_flag;
  const int bn = y.ld % 128 ? 64 : c->opt[SNN_OPT_LAYER_NEURONS];   // 128: 108.0 us per step at 700-128-128-20, 64: 109.7
  // Two workgroups per sample, taking its blocks of 64 steps in turn (SNN_OPT_LAYER_TIME_SPLIT, on
  // request: 29.3 us against 28.8 at 700-128-128-20, T = 128, B = 256): from two blocks on, and while a
  // block count fits the flags' 10 bits.
  const bool split = c->opt[SNN_OPT_LAYER_TIME_SPLIT] && bn == 128 && c->T > 64 && c->T <= 64 * 1000;
  // A pair of layers on two workgroups per sample (SNN_OPT_LAYER_PAIR = 2, on request: 32.9 us against
  // 27.7 at 700-128-128-20, T = 128, B = 256): the upper layer's workgroup follows the lower layer's,
  // 64 steps at a time.
  const bool lsplit = nl == 2 && c->opt[SNN_OPT_LAYER_PAIR] == 2 && !split && c->T <= 64 * 1000;
  if (split || lsplit) {
    if (++c->fwd_epoch >= (1 << 21)) {                // long before the flags' counter wraps: start over
      HIPCHK(c, fill_zero(c->stream, c->hand, rup(c->B, 8) * c->hand_parts * SNN_HAND_BYTES));
      c->fwd_epoch = 1;
    }
    a.hand = c->hand;
    a.epoch = c->fwd_epoch;
  }
  Bracket br(c, SNN_K_LIF_FORWARD, l + 1);
  const dim3 grid((unsigned)(rup(c->B, 8) * (y.ld / bn) * (split || lsplit ? 2 : 1)));
#define SNN_LFWD3(RO, PK, TS_)                                                                                   \
  do {                                                                                                           \
    if (lsplit) hipLaunchKernelGGL((lif_layer_forward_kernel<2, 3, RO, 2, PK, 1, 2>), grid, dim3(256), 0, c->stream, a); \
    else if (nl == 2) hipLaunchKernelGGL((lif_layer_forward_kernel<2, 3, RO, 2, PK, TS_>), grid, dim3(256), 0, c->stream, a); \
    else hipLaunchKernelGGL((lif_layer_forward_kernel<2, 3, RO, 1, PK, TS_>), grid, dim3(256), 0, c->stream, a); \
  } while (0)
#define SNN_LFWD2(RO, PK) do { if (split) SNN_LFWD3(RO, PK, 2); else SNN_LFWD3(RO, PK, 1); } while (0)
#define SNN_LFWD(RO) do { if (packed) SNN_LFWD2(RO, true); else SNN_LFWD2(RO, false); } while (0)
  if (with_readout) {
    Layer &ro = c->layers[c->L - 1];
    a.J = ro.I; a.ldj = c->ldC; a.Qr = ro.Qf; a.ldqr = ro.ldqf; a.qr_bytes = (unsigned)(ro.qf_plane * 2);
    if (with_readout == 2) {
      if (!labels) return fail(c, SNN_ERR_NULL, "labels are NULL");
      a.Y = ro.V; a.z = c->z; a.tstar = c->tstar; a.labels = labels; a.loss_b = c->loss_b; a.dz = c->dz;
      a.dJ = ro.dI; a.beta_r = ro.beta_v; a.C = c->C;
      if (c->integral) SNN_LFWD(3); else SNN_LFWD(2);
      c->dj_ready = true;
      c->loss_ready = false;
    } else {
      SNN_LFWD(1);
    }
    ro.i_ready = true;
  } else if (bn == 64) {
    if (packed) hipLaunchKernelGGL((lif_layer_forward_kernel<1, 3, 0, 1, true>), grid, dim3(256), 0, c->stream, a);
    else hipLaunchKernelGGL((lif_layer_forward_kernel<1, 3>), grid, dim3(256), 0, c->stream, a);
  } else SNN_LFWD(0);
#undef SNN_LFWD
#undef SNN_LFWD2
#undef SNN_LFWD3
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

int launch_readout_forward(snn_ctx *c, const int32_t *labels) {
  if (!labels) return fail(c, SNN_ERR_NULL, "labels are NULL");
  Layer &y = c->layers[c->L - 1];
  Bracket br(c, SNN_K_READOUT_FORWARD, c->L);
  if (c->ldC <= 64) {
    const int cw = c->ldC <= 16 ? 16 : c->ldC <= 32 ? 32 : 64;
    dim3 grid((c->B + 64 / cw - 1) / (64 / cw)), block(512);
#define SNN_RDL(CW, HL)                                                                                          \
  do {                                                                                                           \
    if (c->integral)                                                                                             \
      hipLaunchKernelGGL((readout_loss_kernel<CW, HL, true>), grid, block, 0, c->stream, y.I, y.V, c->z, c->tstar, \
                         labels, c->loss_b, c->dz, c->err_flag, y.dI, c->T, c->B, c->C, c->ldC, y.beta_v);       \
    else                                                                                                         \
      hipLaunchKernelGGL((readout_loss_kernel<CW, HL, false>), grid, block, 0, c->stream, y.I, y.V, c->z, c->tstar, \
                         labels, c->loss_b, c->dz, c->err_flag, y.dI, c->T, c->B, c->C, c->ldC, y.beta_v);       \
  } while (0)
    if (c->hl) { if (cw == 16) SNN_RDL(16, true); else if (cw == 32) SNN_RDL(32, true); else SNN_RDL(64, true); }
    else { if (cw == 16) SNN_RDL(16, false); else if (cw == 32) SNN_RDL(32, false); else SNN_RDL(64, false); }
#undef SNN_RDL
    HIPCHK(c, hipGetLastError());
    c->dj_ready = true;
    c->loss_ready = false;
    return SNN_OK;
  }
  c->dj_ready = false;
  c->loss_ready = true;
  const int stride = c->B * c->ldC;
  hipLaunchKernelGGL(readout_forward_kernel, dim3((stride + 255) / 256), dim3(256), 0, c->stream, y.I, y.V, c->z,
                     c->tstar, c->T, stride, y.beta_v, c->ldC, c->integral ? 1 : 0);
  HIPCHK(c, hipGetLastError());
  hipLaunchKernelGGL(cross_entropy_kernel, dim3((c->B + 3) / 4), dim3(256), 0, c->stream, c->z, labels, c->loss_b,
                     c->dz, c->B, c->C, c->ldC, c->err_flag);
  HIPCHK(c, hipGetLastError());
  hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(256), 0, c->stream, c->loss_b, c->loss, c->B);
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

int launch_readout_reverse(snn_ctx *c) {
  Layer &y = c->layers[c->L - 1];
  Bracket br(c, SNN_K_READOUT_REVERSE, c->L);
  const int stride = c->B * c->ldC;
  if (c->hl)
    hipLaunchKernelGGL(readout_reverse_kernel<true>, dim3((stride + 255) / 256), dim3(256), 0, c->stream, c->dz,
                       c->tstar, y.dI, c->T, stride, y.beta_v, c->ldC, c->integral ? 1 : 0);
  else
    hipLaunchKernelGGL(readout_reverse_kernel<false>, dim3((stride + 255) / 256), dim3(256), 0, c->stream, c->dz,
                       c->tstar, y.dI, c->T, stride, y.beta_v, c->ldC, c->integral ? 1 : 0);
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

void add_param_job(ParamJobs &jobs, float *W, const float *dW, int K, int N, uint16_t *Qf, int ldqf,
                   long long qf_plane, uint16_t *Qb, int ldqb, long long qb_plane) {
  const int j = jobs.njobs++;
  jobs.W[j] = W; jobs.dW[j] = dW; jobs.K[j] = K; jobs.N[j] = N;
  jobs.Qf[j] = Qf; jobs.ldqf[j] = ldqf; jobs.qf_plane[j] = qf_plane;
  jobs.Qb[j] = Qb; jobs.ldqb[j] = ldqb; jobs.qb_plane[j] = qb_plane;
  jobs.blocks_x[j] = (N + 31) / 32;
  jobs.first_block[j + 1] = jobs.first_block[j] + jobs.blocks_x[j] * ((K + 31) / 32);
}

// SGD (when with_grad) and refresh of the bfloat16 operand planes for layers [l0, l1).
int update_layers(snn_ctx *c, int l0, int l1, bool with_grad, float lr) {
  ParamJobs jobs;
  memset(&jobs, 0, sizeof jobs);
  for (int l = l0; l < l1; ++l) {
    Layer &y = c->layers[l];
    add_param_job(jobs, y.Wm, with_grad ? y.dW : nullptr, y.K, y.N, y.Qf, y.ldqf, y.qf_plane, y.Qb, y.ldqb, y.qb_plane);
    if (y.recurrent)
      add_param_job(jobs, y.Rm, with_grad ? y.dR : nullptr, y.N, y.N, y.QRf, y.ldqr, y.qr_plane, y.QRb, y.ldqr,
                    y.qr_plane);
  }
  hipLaunchKernelGGL(param_update_kernel, dim3(jobs.first_block[jobs.njobs]), dim3(256), 0, c->stream, jobs, lr,
                     c->nplanes);
  HIPCHK(c, hipGetLastError());
  return SNN_OK;
}

// snn_sgd_step right after snn_backward: partial sums -> dW -> W and its operand layouts, one launch.
int reduce_and_update(snn_ctx *c, float lr) {
  ReduceUpdateJobs jobs;
  memset(&jobs, 0, sizeof jobs);
  auto add = [&](float *W, float *dW, int K, int N, uint16_t *Qf, int ldqf, long long qf_plane, uint16_t *Qb, int ldqb,
                 long long qb_plane) {
    const int j = jobs.njobs++;
    jobs.W[j] = W; jobs.dW[j] = dW; jobs.K[j] = K; jobs.N[j] = N;
    jobs.Qf[j] = Qf; jobs.ldqf[j] = ldqf; jobs.qf_plane[j] = qf_plane;
    jobs.Qb[j] = Qb; jobs.ldqb[j] = ldqb; jobs.qb_plane[j] = qb_plane;
    jobs.part[j] = nullptr; jobs.splits[j] = 1;
    for (int r = 0; r < c->pending.njobs; ++r)
      if (c->pending.out[r] == dW) { jobs.part[j] = c->pending.part[r]; jobs.splits[j] = c->pending.splits[r]; }
    jobs.blocks_x[j] = (N + 31) / 32;
    jobs.first_block[j + 1] = jobs.first_block[j] + jobs.blocks_x[j] * ((K + 7) / 8);
  };
  for (int l = 0; l < c->L; ++l) {
    Layer &y = c->layers[l];
    add(y.Wm, y.dW, y.K, y.N, y.Qf, y.ldqf, y.qf_plane, y.Qb, y.ldqb, y.qb_plane);
    if (y.recurrent) add(y.Rm, y.dR, y.N, y.N, y.QRf, y.ldqr, y.qr_plane, y.QRb, y.ldqr, y.qr_plane);
  }
  const bool with_loss = !c->loss_ready;
  hipLaunchKernelGGL(reduce_update_kernel, dim3(jobs.first_block[jobs.njobs] + (with_loss ? 1 : 0)), dim3(256), 0,
                     c->stream, jobs, lr, c->nplanes, with_loss ? c->loss_b : nullptr, c->loss, c->B);
  HIPCHK(c, hipGetLastError());
  if (with_loss) c->loss_ready = true;
  c->reduce_pending = false;
  return SNN_OK;
}

int check_err_flag(snn_ctx *c) {
  int flag = 0;
  HIPCHK(c, hipMemcpyAsync(&flag, c->err_flag, sizeof(int), hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (flag) {
    HIPCHK(c, fill_zero(c->stream, c->err_flag, 256));
    if (flag & 2) return fail(c, SNN_ERR_HIP, "a forward launch gave up waiting for another workgroup");
    return fail(c, SNN_ERR_ARG, "a label was outside [0, C)");
  }
  return SNN_OK;
}

// Describes where a tensor lives: rows x cols elements, leading dimension, element size;
// `hl`: held on the device in hi/lo form, fp32 on the host side.
struct TensorView { void *p; size_t rows, cols, ld, esz; bool hl; };

int view_of(snn_ctx *c, int tensor, int layer, TensorView *v, bool for_set) {
  const size_t M = (size_t)c->M;
  auto spiking_layer = [&](Layer **out) -> int {
    if (layer < 1 || layer > c->L - 1) return fail(c, SNN_ERR_ARG, "layer %d is not a spiking layer", layer);
    *out = &c->layers[layer - 1];
    return SNN_OK;
  };
  auto any_layer = [&](Layer **out) -> int {
    if (layer < 1 || layer > c->L) return fail(c, SNN_ERR_ARG, "layer %d out of range", layer);
    *out = &c->layers[layer - 1];
    return SNN_OK;
  };
  Layer *y = nullptr;
  Layer &ro = c->layers[c->L - 1];
  int rc;
  bool settable = true;
  switch (tensor) {
    case SNN_T_WEIGHT:
      if ((rc = any_layer(&y))) return rc;
      *v = {y->Wm, (size_t)y->K, (size_t)y->N, (size_t)y->N, 4, false}; break;
    case SNN_T_GRAD_W:
      if ((rc = any_layer(&y))) return rc;
      *v = {y->dW, (size_t)y->K, (size_t)y->N, (size_t)y->N, 4, false}; settable = false; break;
    case SNN_T_RWEIGHT:
    case SNN_T_GRAD_R:
      if ((rc = spiking_layer(&y))) return rc;
      if (!y->recurrent) return fail(c, SNN_ERR_ARG, "layer %d is not recurrent", layer);
      *v = {tensor == SNN_T_RWEIGHT ? y->Rm : y->dR, (size_t)y->N, (size_t)y->N, (size_t)y->N, 4, false};
      settable = tensor == SNN_T_RWEIGHT;
      break;
    case SNN_T_BETA:
    case SNN_T_GRAD_BETA:
      if ((rc = any_layer(&y))) return rc;
      if (tensor == SNN_T_GRAD_BETA && !c->learn_beta) return fail(c, SNN_ERR_STATE, "decays are not trained (learn_beta = 0)");
      *v = {tensor == SNN_T_BETA ? y->beta_v : y->dbeta, 1, (size_t)y->N, (size_t)y->ld, 4, false};
      settable = tensor == SNN_T_BETA;
      break;
    case SNN_T_CURRENT:
      if ((rc = spiking_layer(&y))) return rc;
      *v = {y->I, M, (size_t)y->N, (size_t)y->ld, 4, false}; break;
    case SNN_T_MEMBRANE:
      if ((rc = spiking_layer(&y))) return rc;
      *v = {y->V, M, (size_t)y->N, (size_t)y->ld, 4, false}; break;
    case SNN_T_SPIKES:
      if ((rc = spiking_layer(&y))) return rc;
      *v = {y->S, M, (size_t)y->N, (size_t)y->ld, 1, false}; break;
    case SNN_T_ADAPTATION:
      if ((rc = spiking_layer(&y))) return rc;
      if (!y->adaptive) return fail(c, SNN_ERR_ARG, "layer %d has no adaptive threshold", layer);
      *v = {y->A, M, (size_t)y->N, (size_t)y->ld, 4, false}; break;
    case SNN_T_D_SPIKES:
      if ((rc = spiking_layer(&y))) return rc;
      *v = {y->dS, M, (size_t)y->N, (size_t)y->ld, 4, false}; break;
    case SNN_T_D_CURRENT:
      if ((rc = spiking_layer(&y))) return rc;
      *v = {y->dI, M, (size_t)y->N, (size_t)y->ld, 4, c->hl}; break;
    case SNN_T_READOUT_CURRENT: *v = {ro.I, M, (size_t)c->C, (size_t)c->ldC, 4, false}; break;
    case SNN_T_READOUT_TRACE: *v = {ro.V, M, (size_t)c->C, (size_t)c->ldC, 4, false}; settable = false; break;
    case SNN_T_LOGITS: *v = {c->z, (size_t)c->B, (size_t)c->C, (size_t)c->ldC, 4, false}; settable = false; break;
    case SNN_T_ARGMAX_T: *v = {c->tstar, (size_t)c->B, (size_t)c->C, (size_t)c->ldC, 4, false}; break;
    case SNN_T_D_LOGITS: *v = {c->dz, (size_t)c->B, (size_t)c->C, (size_t)c->ldC, 4, false}; break;
    case SNN_T_D_READOUT_CURRENT: *v = {ro.dI, M, (size_t)c->C, (size_t)c->ldC, 4, c->hl}; break;
    case SNN_T_LOSS: *v = {c->loss, 1, 1, 1, 4, false}; settable = false; break;
    case SNN_T_LOSS_PER_SAMPLE: *v = {c->loss_b, 1, (size_t)c->B, (size_t)c->B, 4, false}; settable = false; break;
    default: return fail(c, SNN_ERR_ARG, "unknown tensor id %d", tensor);
  }
  if (for_set && !settable) return fail(c, SNN_ERR_ARG, "tensor %d cannot be set", tensor);
  return SNN_OK;
}

// Host-side twin of the device's hi/lo form (used only to move tensors in and out).
inline uint16_t host_bf16(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
inline float host_bf16_value(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

}  // namespace

// ====================================================================== C ABI
extern "C" {

int32_t snn_workspace_bytes(const snn_config *cfg, size_t *bytes) {
  int rc = validate(cfg);
  if (rc) return rc;
  if (!bytes) return fail(nullptr, SNN_ERR_NULL, "bytes is NULL");
  snn_ctx tmp;
  configure(tmp, cfg);
  Carver cv(nullptr);
  carve(tmp, cv);
  *bytes = cv.off;
  return SNN_OK;
}

int32_t snn_init(const snn_config *cfg, void *workspace_dev, size_t workspace_bytes, const float *const *W_host,
                 const float *const *R_host, void *hip_stream, snn_ctx **out) {
  int rc = validate(cfg);
  if (rc) return rc;
  if (!workspace_dev || !W_host || !out) return fail(nullptr, SNN_ERR_NULL, "workspace, W_host or out is NULL");
  if ((uintptr_t)workspace_dev % 256 != 0) return fail(nullptr, SNN_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  snn_ctx *c = new snn_ctx();
  configure(*c, cfg);
  Carver cv((char *)workspace_dev);
  carve(*c, cv);
  if (cv.off > workspace_bytes) {
    delete c;
    return fail(nullptr, SNN_ERR_WORKSPACE, "workspace too small: need %zu bytes, got %zu", cv.off, workspace_bytes);
  }
  for (int l = 0; l < c->L; ++l) {
    if (!W_host[l]) { delete c; return fail(nullptr, SNN_ERR_NULL, "W_host[%d] is NULL", l); }
    if (c->layers[l].recurrent && (!R_host || !R_host[l])) {
      delete c;
      return fail(nullptr, SNN_ERR_NULL, "R_host[%d] is NULL for a recurrent layer", l);
    }
  }
  c->ws = (char *)workspace_dev; c->ws_bytes = cv.off;
  c->stream = (hipStream_t)hip_stream;
  auto bail = [&](hipError_t e, const char *what) {
    fail(nullptr, SNN_ERR_HIP, "%s failed: %s", what, hipGetErrorString(e));
    delete c;
    return (int32_t)SNN_ERR_HIP;
  };
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess || ndev == 0) return bail(e != hipSuccess ? e : hipErrorNoDevice, "hipGetDeviceCount");
  {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
      c->wall_khz = khz;
    int cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      c->cus = cus;
  }
  {
    void *unused = nullptr;                              // set-up of snn_weight_grad_static on this device
    if ((e = static_scratch(&unused)) != hipSuccess) return bail(e, "hipGetSymbolAddress(scratch)");
  }
  if ((e = hipMemsetAsync(c->ws, 0, c->ws_bytes, c->stream)) != hipSuccess) return bail(e, "hipMemsetAsync(workspace)");
  std::vector<std::vector<float>> beta_host(c->L);        // alive until the synchronisation below
  for (int l = 0; l < c->L; ++l) {
    Layer &y = c->layers[l];
    beta_host[l].assign(y.N, y.beta);
    if ((e = hipMemcpyAsync(y.beta_v, beta_host[l].data(), sizeof(float) * y.N, hipMemcpyHostToDevice, c->stream)) != hipSuccess)
      return bail(e, "hipMemcpyAsync(beta)");
    if ((e = hipMemcpyAsync(y.Wm, W_host[l], sizeof(float) * y.K * y.N, hipMemcpyHostToDevice, c->stream)) != hipSuccess)
      return bail(e, "hipMemcpyAsync(W)");
    if (y.recurrent &&
        (e = hipMemcpyAsync(y.Rm, R_host[l], sizeof(float) * y.N * y.N, hipMemcpyHostToDevice, c->stream)) != hipSuccess)
      return bail(e, "hipMemcpyAsync(R)");
  }
  if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail(e, "hipStreamSynchronize");
  if (update_layers(c, 0, c->L, false, 0.f) != SNN_OK) { g_err = c->err; delete c; return SNN_ERR_HIP; }
  if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail(e, "hipStreamSynchronize");
  *out = c;
  return SNN_OK;
}

// Whether the forward pass runs layer 1 as one launch (the rule of forward_layers below).
static bool first_layer_runs_whole(snn_ctx *c) {
  const int whole = layer_fuse_mode(c);
  const bool whole_top = whole >= 2 && layer_forward_fusable(c, c->L - 2);
  return whole >= 1 && (0 < c->L - 2 || whole_top) && layer_forward_fusable(c, 0);
}

static int32_t forward_layers(snn_ctx *c, const int32_t *labels_dev, float *loss_host) {
  int rc;
  const int whole = layer_fuse_mode(c);                 // layers that run as one launch, product and scan
  const bool whole_top = whole >= 2 && layer_forward_fusable(c, c->L - 2);
  const int with_readout = whole_top ? layer_forward_takes_readout(c) : 0;
  const bool fuse_top = !whole_top && top_forward_fusable(c);   // the last spiking layer's scan forms the readout's currents
  for (int l = 0; l < c->L; ++l) {
    if (whole >= 1 && (l < c->L - 2 || whole_top) && layer_forward_fusable(c, l)) {
      // this layer and the next in one launch when both hold exactly 128 padded neurons
      // (SNN_OPT_LAYER_PAIR = 0: one launch each)
      const bool pair = c->opt[SNN_OPT_LAYER_PAIR] && c->opt[SNN_OPT_LAYER_NEURONS] == 128 && c->layers[l].ld == 128 && l + 1 <= c->L - 2 &&
                        (l + 1 < c->L - 2 || whole_top) && layer_forward_fusable(c, l + 1) && c->layers[l + 1].ld == 128;
      const int nl = pair ? 2 : 1;
      if ((rc = launch_layer_forward(c, l, nl, l + nl - 1 == c->L - 2 ? with_readout : 0, labels_dev))) return rc;
      l += nl - 1;
      continue;
    }
    if (l == c->L - 1 && with_readout) {                // J is there already, perhaps the whole readout
      if (with_readout == 1 && (rc = launch_readout_forward(c, labels_dev))) return rc;
      continue;
    }
    if (!(fuse_top && l == c->L - 1) && (rc = launch_current_gemm(c, l))) return rc;
    if (c->layers[l].spiking) {
      if ((rc = fuse_top && l == c->L - 2 ? launch_lif_forward_top(c) : launch_lif_forward(c, l))) return rc;
    } else {
      if ((rc = launch_readout_forward(c, labels_dev))) return rc;
    }
  }
  c->state = 1;
  if (loss_host) {
    if ((rc = ensure_loss(c))) return rc;
    HIPCHK(c, hipMemcpyAsync(loss_host, c->loss, sizeof(float), hipMemcpyDeviceToHost, c->stream));
    if ((rc = check_err_flag(c))) return rc;
  }
  return SNN_OK;
}

int32_t snn_forward(snn_ctx *c, const uint8_t *x_dev, const int32_t *labels_dev, float *loss_host) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (!x_dev || !labels_dev) return fail(c, SNN_ERR_NULL, "x_dev or labels_dev is NULL");
  c->labels_dev = labels_dev;
  int rc;
  if ((rc = prepare_input(c, x_dev))) return rc;
  return forward_layers(c, labels_dev, loss_host);
}

int32_t snn_forward_packed(snn_ctx *c, const uint8_t *x_packed_dev, const int32_t *labels_dev, float *loss_host) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (!x_packed_dev || !labels_dev) return fail(c, SNN_ERR_NULL, "x_packed_dev or labels_dev is NULL");
  c->labels_dev = labels_dev;
  int rc;
  // Where layer 1 runs as one launch, that launch (and the weight-gradient launch) reads the packed
  // raster itself: rows of a multiple of 4 bytes, at most 1024 channels.  Otherwise the raster is
  // unpacked into the workspace first.
  c->x_packed = x_packed_dev;
  c->x_direct = c->sizes[0] % 4 == 0 && c->sizes[0] <= 1024 && (uintptr_t)x_packed_dev % 4 == 0 && first_layer_runs_whole(c);
  c->x_unpacked = false;
  if (c->x_direct) c->x_eff = nullptr;
  else if ((rc = prepare_packed_input(c, x_packed_dev))) return rc;
  return forward_layers(c, labels_dev, loss_host);
}

int32_t snn_backward(snn_ctx *c) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (c->state < 1) return fail(c, SNN_ERR_STATE, "snn_backward needs a preceding snn_forward");
  int rc;
  ReduceJobs jobs;
  memset(&jobs, 0, sizeof jobs);
  WgradJobs wj;
  memset(&wj, 0, sizeof wj);
  if (!c->dj_ready && (rc = launch_readout_reverse(c))) return rc;
  for (int l = c->L - 1; l >= 0; --l) {
    const bool fused = reverse_fusable(c, l);           // this layer's scan forms its own dS
    if (c->layers[l].spiking) {
      c->layers[l].ds_ready = !fused;
      if ((rc = fused ? launch_lif_reverse_fused(c, l) : launch_lif_reverse(c, l))) return rc;
    }
    if (l == 0 && c->prof.cls == SNN_K_EVENT_PAIR) { Bracket br(c, SNN_K_EVENT_PAIR, 0); }
    if (l == 0 && c->prof.cls == SNN_K_CALIBRATE) {
      Bracket br(c, SNN_K_CALIBRATE, 0);
      hipLaunchKernelGGL(wait_ticks_kernel, dim3(1), dim3(64), 0, c->stream,
                         (long long)c->wall_khz * SNN_CALIBRATE_US / 1000, (long long *)c->err_flag + 8);
      HIPCHK(c, hipGetLastError());
    }
    if ((rc = queue_weight_grad(c, l, wj, jobs))) return rc;
    if (l > 0 && !reverse_fusable(c, l - 1) && (rc = launch_input_grad(c, l))) return rc;
  }
  if (c->learn_beta) {
    // per-sample parts of dL/dbeta: written by the reverse scans for the spiking layers, by a
    // kernel of its own for the readout; summed over the batch by the reduction launch
    Layer &ro = c->layers[c->L - 1];
    const int stride = c->B * c->ldC;
    if (c->hl)
      hipLaunchKernelGGL(readout_beta_grad_kernel<true>, dim3((stride + 255) / 256), dim3(256), 0, c->stream, ro.dI,
                         ro.V, ro.part_b, c->T, stride);
    else
      hipLaunchKernelGGL(readout_beta_grad_kernel<false>, dim3((stride + 255) / 256), dim3(256), 0, c->stream, ro.dI,
                         ro.V, ro.part_b, c->T, stride);
    HIPCHK(c, hipGetLastError());
    for (int l = 0; l < c->L; ++l)
      if (!add_reduce_job(jobs, c->layers[l].part_b, c->layers[l].dbeta, c->B, c->layers[l].ld, true))
        return fail(c, SNN_ERR_UNSUPPORTED, "more than %d gradient reductions in one backward pass", SNN_MAX_REDUCE_JOBS);
  }
  // Without trained decays the reduction of the partial sums waits for snn_sgd_step, which does
  // it in the launch that updates the parameters (SNN_OPT_DEFER_REDUCE = 0: reduce here).
  const bool defer = !c->learn_beta && c->opt[SNN_OPT_DEFER_REDUCE];
  if ((rc = launch_weight_grads(c, wj, jobs, !c->loss_ready, defer))) return rc;
  c->state = 2;
  return SNN_OK;
}

int32_t snn_sgd_step(snn_ctx *c, float lr) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (c->state < 2) return fail(c, SNN_ERR_STATE, "snn_sgd_step needs a preceding snn_backward");
  Bracket br(c, SNN_K_SGD, 0);
  int rc = c->reduce_pending ? reduce_and_update(c, lr) : update_layers(c, 0, c->L, true, lr);
  if (rc) return rc;
  if (c->learn_beta) {
    BetaJobs bj;
    memset(&bj, 0, sizeof bj);
    for (int l = 0; l < c->L; ++l) {
      const int j = bj.njobs++;
      bj.beta[j] = c->layers[l].beta_v; bj.dbeta[j] = c->layers[l].dbeta;
      bj.first[j + 1] = bj.first[j] + c->layers[l].N;
    }
    hipLaunchKernelGGL(beta_update_kernel, dim3((bj.first[bj.njobs] + 255) / 256), dim3(256), 0, c->stream, bj, lr);
    HIPCHK(c, hipGetLastError());
  }
  c->state = 0;
  return SNN_OK;
}

int32_t snn_get_tensor(snn_ctx *c, int32_t tensor, int32_t layer, void *dst, size_t bytes) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (!dst) return fail(c, SNN_ERR_NULL, "dst_host is NULL");
  TensorView v;
  int rc = view_of(c, tensor, layer, &v, false);
  if (rc) return rc;
  if (bytes != v.rows * v.cols * v.esz)
    return fail(c, SNN_ERR_SHAPE, "tensor %d needs %zu bytes, got %zu", tensor, v.rows * v.cols * v.esz, bytes);
  if ((rc = flush_reduce(c))) return rc;
  if (tensor == SNN_T_LOSS && (rc = ensure_loss(c))) return rc;
  if (tensor == SNN_T_CURRENT && layer >= 1 && layer <= c->L - 1 && !c->layers[layer - 1].i_ready) {
    if ((rc = launch_current_gemm(c, layer - 1))) return rc;   // the layer ran as one launch: materialise I now
  }
  if (tensor == SNN_T_D_SPIKES && layer >= 1 && layer <= c->L - 1 && !c->layers[layer - 1].ds_ready) {
    if ((rc = launch_input_grad(c, layer))) return rc;   // formed on the fly in snn_backward: materialise it now
    c->layers[layer - 1].ds_ready = true;
  }
  HIPCHK(c, hipMemcpy2DAsync(dst, v.cols * v.esz, v.p, v.ld * v.esz, v.cols * v.esz, v.rows, hipMemcpyDeviceToHost,
                             c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (v.hl) {                                   // hi + lo -> fp32, in place
    uint32_t *w = (uint32_t *)dst;
    float *f = (float *)dst;
    for (size_t i = 0; i < v.rows * v.cols; ++i)
      f[i] = host_bf16_value((uint16_t)(w[i] & 0xFFFFu)) + host_bf16_value((uint16_t)(w[i] >> 16));
  }
  return check_err_flag(c);
}

int32_t snn_set_tensor(snn_ctx *c, int32_t tensor, int32_t layer, const void *src, size_t bytes) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (!src) return fail(c, SNN_ERR_NULL, "src_host is NULL");
  TensorView v;
  int rc = view_of(c, tensor, layer, &v, true);
  if (rc) return rc;
  if (bytes != v.rows * v.cols * v.esz)
    return fail(c, SNN_ERR_SHAPE, "tensor %d needs %zu bytes, got %zu", tensor, v.rows * v.cols * v.esz, bytes);
  if (tensor == SNN_T_BETA) {
    const float *f = (const float *)src;
    for (size_t i = 0; i < v.cols; ++i)
      if (!(f[i] >= 0.f && f[i] <= 1.f)) return fail(c, SNN_ERR_ARG, "beta[%zu] outside [0,1]", i);
  }
  std::vector<uint32_t> tmp;
  if (v.hl) {                                   // fp32 -> hi/lo words
    const float *f = (const float *)src;
    tmp.resize(v.rows * v.cols);
    for (size_t i = 0; i < tmp.size(); ++i) {
      const uint16_t h = host_bf16(f[i]);
      const uint16_t l = host_bf16(f[i] - host_bf16_value(h));
      tmp[i] = (uint32_t)h | ((uint32_t)l << 16);
    }
    src = tmp.data();
  }
  HIPCHK(c, hipMemcpy2DAsync(v.p, v.ld * v.esz, src, v.cols * v.esz, v.cols * v.esz, v.rows, hipMemcpyHostToDevice,
                             c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (tensor == SNN_T_D_LOGITS || tensor == SNN_T_ARGMAX_T) c->dj_ready = false;   // dJ must be recomputed
  if (tensor == SNN_T_CURRENT) c->layers[layer - 1].i_ready = true;     // what the caller imposed is what a reader gets
  if (tensor == SNN_T_D_SPIKES) c->layers[layer - 1].ds_ready = true;
  if (tensor == SNN_T_BETA) c->state = 0;                               // a forward pass on other decays is stale
  if (tensor == SNN_T_WEIGHT || tensor == SNN_T_RWEIGHT) {
    if ((rc = update_layers(c, layer - 1, layer, false, 0.f))) return rc;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->state = 0;
  }
  return SNN_OK;
}

int32_t snn_run_step(snn_ctx *c, int32_t step, int32_t layer, const uint8_t *x_dev, const int32_t *labels_dev) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (layer < 1 || layer > c->L) return fail(c, SNN_ERR_ARG, "layer %d out of range", layer);
  const int l = layer - 1;
  const bool spiking = c->layers[l].spiking;
  {
    int rc = flush_reduce(c);
    if (rc) return rc;
  }
  if (x_dev) {
    int rc = prepare_input(c, x_dev);
    if (rc) return rc;
  }
  switch (step) {
    case SNN_STEP_CURRENT_GEMM: return launch_current_gemm(c, l);
    case SNN_STEP_LIF_FORWARD:
      if (!spiking) return fail(c, SNN_ERR_ARG, "layer %d is not spiking", layer);
      return launch_lif_forward(c, l);
    case SNN_STEP_READOUT_FORWARD: return launch_readout_forward(c, labels_dev);
    case SNN_STEP_READOUT_REVERSE: return launch_readout_reverse(c);
    case SNN_STEP_LIF_REVERSE:
      if (!spiking) return fail(c, SNN_ERR_ARG, "layer %d is not spiking", layer);
      return launch_lif_reverse(c, l);
    case SNN_STEP_WEIGHT_GRAD: {
      ReduceJobs jobs;
      memset(&jobs, 0, sizeof jobs);
      WgradJobs wj;
      memset(&wj, 0, sizeof wj);
      int rc = queue_weight_grad(c, l, wj, jobs);
      return rc ? rc : launch_weight_grads(c, wj, jobs, false);
    }
    case SNN_STEP_INPUT_GRAD:
      if (l == 0) return fail(c, SNN_ERR_ARG, "layer 1 has no input gradient");
      return launch_input_grad(c, l);
    default: return fail(c, SNN_ERR_ARG, "unknown step %d", step);
  }
}

int32_t snn_weight_grad_static(const uint8_t *S_dev, const float *G_dev, float *dW_dev, int64_t M, int32_t K, int32_t N,
                               void *hip_stream) {
  if (!S_dev || !G_dev || !dW_dev) return fail(nullptr, SNN_ERR_NULL, "S_dev, G_dev or dW_dev is NULL");
  if (M <= 0 || K <= 0 || N <= 0) return fail(nullptr, SNN_ERR_ARG, "M, K and N must be positive");
  if (K % 4 || N % 4) return fail(nullptr, SNN_ERR_ARG, "K and N must be multiples of 4");
  if ((uintptr_t)S_dev % 4 || (uintptr_t)G_dev % 16 || (uintptr_t)dW_dev % 16)
    return fail(nullptr, SNN_ERR_ARG, "S_dev must be 4-byte aligned, G_dev and dW_dev 16-byte aligned");
  if (M > SNN_STATIC_MAX_ROWS || (long long)K * N > SNN_STATIC_MAX_WEIGHTS || M * K >= (1ll << 31) || M * N * 4 >= (1ll << 31))
    return fail(nullptr, SNN_ERR_UNSUPPORTED,
                "beyond the static scratch: M <= %d, K * N <= %d, M * K < 2^31 and M * N * 4 < 2^31 are required",
                SNN_STATIC_MAX_ROWS, SNN_STATIC_MAX_WEIGHTS);
  hipStream_t st = (hipStream_t)hip_stream;
  void *scr = nullptr;
  hipError_t e = static_scratch(&scr);
  if (e != hipSuccess) return fail(nullptr, SNN_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
  // Splits as for a context's products, but no more than fit the scratch (a single split needs
  // none: it writes dW itself).  Every split writes its whole K x N slice before the reduction
  // reads it, so nothing has to be cleared between calls.
  const long long weights = (long long)K * N;
  long long per = 0;
  int splits = choose_splits(M, wgrad_tiles(K, N, false), weights, K + 4ll * N, &per, false);
  const long long fit = (long long)SNN_STATIC_SCRATCH_BYTES / (weights * 4);
  if (splits > fit) {
    per = (long long)rup((size_t)((M + fit - 1) / fit), 64);
    splits = (int)((M + per - 1) / per);
  }
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.P = S_dev; a.ldp = K; a.p_ivalid = K; a.p_bytes = (unsigned)(M * K);
  a.Q = G_dev; a.ldq = N; a.q_bytes = (unsigned)(M * N * 4);
  a.rows = K; a.cols = N; a.ldc = N; a.kc = (int)M;
  a.kc_per_split = (int)per;
  a.c_split_stride = weights;
  a.C = splits > 1 ? (float *)scr : dW_dev;
  GemmJobs jobs;
  memset(&jobs, 0, sizeof jobs);
  if (N <= 32) {
    gemm_jobs_add<4, 1, 1, 1>(jobs, a, splits);
    e = gemm_jobs_launch<P_T_U8, Q_T_F32S, EPI_STORE, 4, 1, 1, 1, 3, 1>(jobs, st);
  } else if (N <= 64) {
    gemm_jobs_add<2, 2, 2, 1>(jobs, a, splits);
    e = gemm_jobs_launch<P_T_U8, Q_T_F32S, EPI_STORE, 2, 2, 2, 1, 3, 1>(jobs, st);
  } else {
    gemm_jobs_add<2, 2, 2, 2>(jobs, a, splits);
    e = gemm_jobs_launch<P_T_U8, Q_T_F32S, EPI_STORE, 2, 2, 2, 2, 3, 1>(jobs, st);
  }
  if (e != hipSuccess) return fail(nullptr, SNN_ERR_HIP, "weight-gradient launch failed: %s", hipGetErrorString(e));
  if (splits > 1) {
    ReduceJobs red;
    memset(&red, 0, sizeof red);
    add_reduce_job(red, (const float *)scr, dW_dev, splits, weights);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(red.first_block[1]), dim3(256), 0, st, red, nullptr, nullptr, 0);
    if ((e = hipGetLastError()) != hipSuccess)
      return fail(nullptr, SNN_ERR_HIP, "reduction launch failed: %s", hipGetErrorString(e));
  }
  return SNN_OK;
}

int32_t snn_set_option(snn_ctx *c, int32_t option, int32_t value) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  bool ok;
  switch (option) {
    case SNN_OPT_LAYER_FORWARD: ok = value >= 0 && value <= 4; break;
    case SNN_OPT_LAYER_REVERSE:
    case SNN_OPT_LAYER_PAIR: ok = value >= 0 && value <= 2; break;
    case SNN_OPT_LAYER_TIME_SPLIT:
    case SNN_OPT_TOP_SCANS:
    case SNN_OPT_WGRAD_TR:
    case SNN_OPT_RLIF_PERSIST:
    case SNN_OPT_WAIT_FAULT:
    case SNN_OPT_DEFER_REDUCE:
    case SNN_OPT_STREAM_GEMM: ok = value == 0 || value == 1; break;
    case SNN_OPT_LAYER_MIN_BATCH: ok = value >= 0; break;
    case SNN_OPT_WAIT_LIMIT_LOG2: ok = value >= 4 && value <= 20; break;
    case SNN_OPT_LAYER_NEURONS: ok = value == 64 || value == 128; break;
    case SNN_OPT_LAYER_MAX_NEURONS: ok = value >= 64 && value <= 1024; break;
    case SNN_OPT_STREAM_MIN_MB: ok = value >= 0 && value <= (1 << 20); break;
    case SNN_OPT_TILE_ROWS: ok = value == 0 || value == 32 || value == 64 || value == 128; break;
    default: return fail(c, SNN_ERR_ARG, "unknown option %d", option);
  }
  if (!ok) return fail(c, SNN_ERR_ARG, "value %d is out of range for option %d", value, option);
  c->opt[option] = value;
  return SNN_OK;
}

int32_t snn_get_option(const snn_ctx *c, int32_t option, int32_t *value) {
  if (!c || !value) return fail(nullptr, SNN_ERR_NULL, "context or value is NULL");
  if (option < 0 || option >= SNN_OPT_COUNT) return fail(nullptr, SNN_ERR_ARG, "unknown option %d", option);
  *value = c->opt[option];
  return SNN_OK;
}

int32_t snn_profile_select(snn_ctx *c, int32_t kernel_class, int32_t layer) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (kernel_class < SNN_K_NONE || kernel_class >= SNN_K_COUNT) return fail(c, SNN_ERR_ARG, "unknown kernel class");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->prof.cls = kernel_class; c->prof.layer = layer; c->prof.used = 0; c->prof.seen = 0;
  return SNN_OK;
}

int32_t snn_profile_every(snn_ctx *c, int32_t n) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (n < 1) return fail(c, SNN_ERR_ARG, "n must be at least 1");
  c->prof.every = n;
  c->prof.seen = 0;
  return SNN_OK;
}

int32_t snn_profile_read(snn_ctx *c, double *total_ms, int64_t *launches) {
  if (!c) return fail(nullptr, SNN_ERR_NULL, "context is NULL");
  if (!total_ms || !launches) return fail(c, SNN_ERR_NULL, "output pointer is NULL");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  double sum = 0;
  for (size_t i = 0; i + 1 < c->prof.used; i += 2) {
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, c->prof.ev[i], c->prof.ev[i + 1]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = (int64_t)(c->prof.used / 2);
  c->prof.used = 0;
  return SNN_OK;
}

int32_t snn_destroy(snn_ctx *c) {
  if (!c) return SNN_OK;
  (void)hipStreamSynchronize(c->stream);
  for (hipEvent_t e : c->prof.ev) (void)hipEventDestroy(e);
  delete c;
  return SNN_OK;
}

const char *snn_last_error(const snn_ctx *c) { return c ? c->err.c_str() : g_err.c_str(); }

}  // extern "C"
