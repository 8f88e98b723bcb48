// Learner entry points of the C ABI (include/msrl.h): minibatch gradient of the PPO clipped
// surrogate, Adam, and the update loop of Learner.learn (Listing 1 of the paper).  Host
// orchestration of the kernels in learn_kernels.h; see that file for the arithmetic.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "../../include/msrl.h"
#include "api_common.h"
#include "learn_kernels.h"
#include "learn_fused_aux.h"

using namespace msrl;

namespace {

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// device buffers of one network's pass over a minibatch (element type = compute type); index l is
// the hidden layer, 0 .. layers-1
constexpr int MAX_LAYERS = 8;
struct NetBufs {
  void* wt[MAX_LAYERS];   // forward weights, transposed: [H, Dp] for l = 0, [H, H] above
  void* wn[MAX_LAYERS];   // backward weights, as stored: [H, H] for l >= 1 (inputs x outputs)
  void *wt3, *wn3;        // output layer: [32, H] and [H, 32]
  float* b3;              // output bias padded to 32
  void* h[MAX_LAYERS];    // activations [Rp, H]
  void* ht[MAX_LAYERS];   // ... unit-major [H, Rp] (in the on-chip path: the tiled layout)
  void* dz[MAX_LAYERS];   // dL/d pre-activation [Rp, H] (l >= 1; layer 0 is only needed unit-major)
  void* dzt[MAX_LAYERS];  // ... unit-major
  float* y;               // [Rp, 32]
  void *dy, *dyt;         // [Rp, 32] and unit-major [32, Rp]
};

}  // namespace

struct msrl_learner {
  msrl_policy_cfg pol;
  int layers;            // hidden layers of both networks
  int64_t max_rows, Rp;  // Rp: max_rows rounded up to 128
  int Dp;                // in_dim rounded up to 16
  bool bf16;
  size_t esz;
  void* xc;              // [Rp, Dp]
  void* xt;              // [Dp, Rp]
  // centralised critic: the value network reads groups of G consecutive rows as one input of G * in_dim
  int G;                 // rows per input of the value network (1: the row itself)
  int Dvp;               // G * in_dim rounded up to 16
  void* xcv;             // [Rp / G (+ padding), Dvp]
  void* xtv;             // [Dvp, Rp]
  NetBufs net[2];
  float* grad;           // scratch gradient of msrl_ppo_update
  float* part;           // [part_slices][part_stride]: the slices' shares of a gradient, added up in slice order
  int part_slices;       // most slices any contraction may be split into
  int64_t part_stride;   // n_params rounded up to 64 floats
  float* stats;          // [8 + 5 * STAT_BINS]: results, then the bins the loss kernel adds into
  size_t n_params;
  // on-chip gradient pass (learn_fused.h): bf16 networks with a categorical policy of at most 16 actions
  bool fused;            // ... for both networks
  bool fused_policy;     // ... for the policy network only (centralised critic: its value network takes path (2))
  int kt1;               // layer-1 tiles of the row kernel: inputs, plus the two bias parts, in tiles of 16
  NetLayout fly;         // layout of one image of the packed weights
  uint8_t* fpacked;      // per network: forward image, backward image
  int cus;               // compute units of the device
};

namespace {

#define LTRY(expr)                                                                          \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail(e_ == hipErrorOutOfMemory ? MSRL_ENOMEM : MSRL_EDEVICE, "%s failed: %s",  \
                  #expr, hipGetErrorString(e_));                                            \
  } while (0)

size_t net_count(int in, int H, int out, int layers = 2) {
  return (size_t)in * H + H + (size_t)(layers - 1) * ((size_t)H * H + H) + (size_t)H * out + out;
}

template <typename T> int dev_alloc(T** p, size_t bytes) {
  LTRY(hipMalloc((void**)p, bytes));
  LTRY(hipMemset(*p, 0, bytes));
  return MSRL_OK;
}

dim3 grid1(int64_t n, int block = 256) { return dim3((unsigned)((n + block - 1) / block)); }

// ---- typed launch helpers (C = compute element type)
template <bool BF16> struct CT;
template <> struct CT<true> { typedef __bf16 T; };
template <> struct CT<false> { typedef float T; };

template <bool BF16, typename SC, int EPI>
hipError_t gemm(hipStream_t s, const void* A, int64_t M_alloc, int64_t lda, const void* B, int64_t N_alloc,
                int64_t ldb, void* C, int64_t M, int64_t N, int64_t ldc, int64_t K, const float* bias,
                const void* Hm, int64_t ldh, int slices = 1, int64_t slice_stride = 0, int* used = nullptr) {
  // EPI_PARTIAL: C is the first of `*used` copies, slice_stride floats apart, one per slice of K
  typedef typename CT<BF16>::T E;
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.A = A; g.B = B; g.C = C; g.bias = bias; g.Hm = Hm;
  g.M = M; g.N = N; g.M_alloc = M_alloc; g.N_alloc = N_alloc; g.K = K;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.ldh = ldh;
  const int64_t kt = Frag<BF16>::KT;
  g.k_per_slice = round_up((K + slices - 1) / slices, kt);
  g.slice_stride = slice_stride;
  slices = (int)((K + g.k_per_slice - 1) / g.k_per_slice);  // no empty slice: every copy of C is written
  if (used) *used = slices;
  dim3 grid((unsigned)((M + 127) / 128), (unsigned)((N + 127) / 128), (unsigned)slices);
  hipLaunchKernelGGL((gemm_kernel<BF16, E, E, SC, EPI>), grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

// row-parallel contraction (weights in LDS, optional unit-major copy Ct of the result)
template <bool BF16, typename SC, int EPI, bool WIDE = false>
hipError_t rowgemm(hipStream_t s, const void* A, int64_t M_alloc, int64_t lda, const void* B, int64_t N_alloc,
                   int64_t ldb, void* C, int64_t M, int64_t N, int64_t ldc, int64_t K, const float* bias,
                   const void* Hm, int64_t ldh, void* Ct, int64_t ldt, int64_t M_pad, float* colsum = nullptr,
                   int64_t colsum_stride = 0, int* colsum_slices = nullptr) {
  // colsum: the first of `*colsum_slices` copies (one per workgroup along x), colsum_stride floats apart
  // wide: K in (256, 704], bf16 only (the panel of 64 columns x 704 inputs is 88 KB of LDS)
  constexpr int NT = BF16 && !WIDE ? 4 : 2;
  constexpr int KMAX = WIDE ? 704 : 256;
  static_assert(!WIDE || BF16, "the wide panel exists in bf16 only");
  RowGemmArgs ra;
  memset(&ra, 0, sizeof(ra));
  GemmArgs& g = ra.g;
  g.A = A; g.B = B; g.C = C; g.bias = bias; g.Hm = Hm;
  g.M = M; g.N = N; g.M_alloc = M_alloc; g.N_alloc = N_alloc; g.K = K;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.ldh = ldh;
  ra.Ct = Ct; ra.ldt = ldt; ra.M_pad = Ct ? M_pad : M; ra.colsum = colsum; ra.colsum_stride = colsum_stride;
  ra.tiles = (ra.M_pad + 255) / 256;
  if (colsum_slices) *colsum_slices = (int)(ra.tiles < 256 ? ra.tiles : 256);
  if (K > KMAX || N % 8 != 0) return hipErrorInvalidValue;  // shapes the learner never produces
  dim3 grid((unsigned)((N + 32 * NT - 1) / (32 * NT)), (unsigned)(ra.tiles < 256 ? ra.tiles : 256));
  hipLaunchKernelGGL((rowgemm_kernel<BF16, SC, EPI, NT, KMAX>), grid, dim3(512), 0, s, ra);
  return hipGetLastError();
}

// weight-gradient contraction: C[slice][M <= 256, N <= 256] = A B^T over the slice's part of K = rows; K is split
// into at most `slices` parts, `*used` of them in the end, whose copies of C lie slice_stride floats apart
template <bool BF16>
hipError_t wgrad(hipStream_t s, const void* A, int64_t M_alloc, int64_t lda, const void* B, int64_t N_alloc,
                 int64_t ldb, float* C, int64_t M, int64_t N, int64_t ldc, int64_t K, int slices, int64_t slice_stride,
                 int* used_out) {
  typedef typename CT<BF16>::T E;
  if (M > 256 || N > 256) return hipErrorInvalidValue;
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.A = A; g.B = B; g.C = C;
  g.M = M; g.N = N; g.M_alloc = M_alloc; g.N_alloc = N_alloc; g.K = K;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  const int64_t kc = 4 * Frag<BF16>::KT;
  g.k_per_slice = round_up((K + slices - 1) / slices, kc);
  g.slice_stride = slice_stride;
  const int64_t used = (K + g.k_per_slice - 1) / g.k_per_slice;
  *used_out = (int)used;
  hipLaunchKernelGGL((wgrad_kernel<BF16, E>), dim3((unsigned)used), dim3(512), 0, s, g);
  return hipGetLastError();
}

template <typename S, typename D>
hipError_t transpose(hipStream_t s, const S* src, int64_t rows, int64_t cols, int64_t ld_src, D* dst, int64_t ldd,
                     int64_t rows_pad, int64_t cols_out) {
  dim3 grid((unsigned)((rows_pad + 31) / 32), (unsigned)((cols_out + 31) / 32));
  hipLaunchKernelGGL((transpose_kernel<S, D>), grid, dim3(256), 0, s, src, rows, cols, ld_src, dst, ldd, rows_pad,
                     cols_out);
  return hipGetLastError();
}

template <typename S, typename D>
hipError_t convert_pad(hipStream_t s, const S* src, int64_t rows, int64_t cols, int64_t ld_src, D* dst, int64_t ldd,
                       int64_t rows_pad) {
  hipLaunchKernelGGL((convert_pad_kernel<S, D>), grid1(rows_pad * ldd), dim3(256), 0, s, src, rows, cols, ld_src,
                     dst, ldd, rows_pad);
  return hipGetLastError();
}

// The parameter tensors of a gradient pass, each with the number of slices its contraction was split
// into; launch() adds the slices' copies (in L->part) up into grad, in slice order.
struct Reducer {
  ReduceJobs j;
  int blocks;
  Reducer() : blocks(0) { memset(&j, 0, sizeof(j)); }
  void add(size_t offset, size_t count, int slices) {
    j.offset[j.jobs] = (int32_t)offset;
    j.count[j.jobs] = (int32_t)count;
    j.slices[j.jobs] = slices;
    j.first_block[j.jobs] = blocks;
    blocks += (int)((count + REDUCE_ELEMS - 1) / REDUCE_ELEMS);
    j.first_block[++j.jobs] = blocks;
  }
  // adam: the step to apply to what is summed, or null; stats: bins to add up on the way, or null
  hipError_t launch(const msrl_learner* L, float* grad, const AdamArgs* adam, float* stats, hipStream_t s) {
    if (j.jobs == 0) return hipSuccess;
    AdamArgs none;
    memset(&none, 0, sizeof(none));
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)blocks + (stats ? 1u : 0u)), dim3(256), 0, s,
                       (const float*)L->part, L->part_stride, j, grad, adam ? *adam : none, stats);
    return hipGetLastError();
  }
};
static_assert(REDUCE_MAX_JOBS >= 2 * 2 * (MAX_LAYERS + 1), "a weight and a bias tensor per layer and network");

// gradient of one minibatch; the handled networks' part of grad (device, n_params floats) is overwritten;
// stats[0..4] are sums
template <bool BF16>
int grad_pass(msrl_learner* L, const float* params, int64_t R, const RowSel& sel, const float* obs, const void* actions,
              const float* logp_old, const float* adv, const float* ret, const msrl_ppo_cfg* c, float* grad,
              hipStream_t s, const AdamArgs* adam, int nets = 3, bool finish = true) {
  // nets: bit n set = network n (0 policy, 1 value) is handled here; with bit 0 clear, the statistics bins
  // have been cleared by the caller and the on-chip pass adds the policy network's part.
  // finish: add the statistics bins up at the end (not while another pass still adds to them)
  typedef typename CT<BF16>::T E;
  const int H = L->pol.hidden;
  const int64_t Rp = L->Rp;
  // per network: input width, its padded width, rows and rows as a contraction length, inputs in
  // compute type row-major and unit-major.  A centralised critic (G > 1) reads G consecutive
  // observation rows as one input: the same memory, seen as [R / G, G * in_dim].
  const int G = L->G;
  const int Dn[2] = {L->pol.in_dim, G * L->pol.in_dim}, Dpn[2] = {L->Dp, G > 1 ? L->Dvp : L->Dp};
  const int64_t Rn[2] = {R, R / G}, Rkn[2] = {round_up(R, 16), round_up(R / G, 16)};
  void* xcn[2] = {L->xc, G > 1 ? L->xcv : L->xc};
  void* xtn[2] = {L->xt, G > 1 ? L->xtv : L->xt};
  if (nets & 1)
    hipLaunchKernelGGL(fill_kernel, grid1(8 + 5 * STAT_BINS), dim3(256), 0, s, L->stats, (int64_t)(8 + 5 * STAT_BINS), 0.0f);
  // observations in compute type, padded; and unit-major
  for (int n = 0; n < (G > 1 ? 2 : 1); ++n) {
    if (!((nets >> n) & 1) && G > 1) continue;
    // (the value network of a centralised critic reads whole groups: the same rows as [R / G, G * in_dim];
    // a selection of rows is refused for it, so only a row offset at a group boundary remains)
    const RowSel rs = n == 0 ? sel : RowSel{sel.row0 / G, 0, 0, 0};
    {
      dim3 grid((unsigned)((Rkn[n] + 63) / 64), (unsigned)((Dpn[n] + 63) / 64));  // (padded sizes: all even)
      hipLaunchKernelGGL((gather_pad_transpose_kernel<E>), grid, dim3(256), 0, s, obs, rs, Rn[n], (int64_t)Dn[n],
                         (int64_t)Dn[n], (E*)xcn[n], (int64_t)Dpn[n], (E*)xtn[n], Rp, Rkn[n]);
      LTRY(hipGetLastError());
    }
  }
  const int NL = L->layers;
  const size_t mid = (size_t)H * H + H;
  const float* P = params;
  for (int n = 0; n < 2; ++n) {
    NetBufs& b = L->net[n];
    const int O = n == 0 ? L->pol.out_dim : 1;
    const int D = Dn[n], Dp = Dpn[n];
    const int64_t R = Rn[n], Rk = Rkn[n];
    const size_t first = (size_t)D * H + H;
    const float* W3 = P + first + (size_t)(NL - 1) * mid;
    const float* b3 = W3 + (size_t)H * O;
    if (!((nets >> n) & 1)) {
      P = b3 + O;
      continue;
    }
    // weights in compute type: transposed for the forward pass, as stored for the backward pass
    LTRY(transpose(s, P, D, H, H, (E*)b.wt[0], Dp, Dp, H));
    for (int l = 1; l < NL; ++l) {
      const float* Wl = P + first + (size_t)(l - 1) * mid;
      LTRY(transpose(s, Wl, H, H, H, (E*)b.wt[l], H, H, H));
      LTRY(convert_pad(s, Wl, H, H, H, (E*)b.wn[l], H, H));
    }
    LTRY(transpose(s, W3, H, O, O, (E*)b.wt3, H, H, 32));
    LTRY(convert_pad(s, W3, H, O, O, (E*)b.wn3, 32, H));
    LTRY(convert_pad(s, b3, 1, O, O, b.b3, 32, 1));
    // forward (the activations also leave unit-major, for the weight gradients)
    if (Dp <= 256) {
      LTRY((rowgemm<BF16, E, EPI_BIAS_TANH>(s, xcn[n], Rp, Dp, b.wt[0], H, Dp, b.h[0], R, H, H, Dp, P + (size_t)D * H, nullptr, 0, b.ht[0], Rp, Rk)));
    } else if (BF16 && Dp <= 704) {
      // the joint observation: the row kernel with a panel of fewer columns and more inputs
      if constexpr (BF16)
        LTRY((rowgemm<BF16, E, EPI_BIAS_TANH, true>(s, xcn[n], Rp, Dp, b.wt[0], H, Dp, b.h[0], R, H, H, Dp, P + (size_t)D * H, nullptr, 0, b.ht[0], Rp, Rk)));
    } else {
      // wider than the row kernel's weight panels: the general kernel, then the unit-major copy
      LTRY((gemm<BF16, E, EPI_BIAS_TANH>(s, xcn[n], Rk, Dp, b.wt[0], H, Dp, b.h[0], R, H, H, Dp, P + (size_t)D * H, nullptr, 0)));
      LTRY(transpose(s, (const E*)b.h[0], R, H, H, (E*)b.ht[0], Rp, Rk, H));
    }
    for (int l = 1; l < NL; ++l) {
      const float* bl = P + first + (size_t)(l - 1) * mid + (size_t)H * H;
      LTRY((rowgemm<BF16, E, EPI_BIAS_TANH>(s, b.h[l - 1], Rp, H, b.wt[l], H, H, b.h[l], R, H, H, H, bl, nullptr, 0, b.ht[l], Rp, Rk)));
    }
    LTRY((gemm<BF16, float, EPI_BIAS>(s, b.h[NL - 1], Rp, H, b.wt3, 32, H, b.y, R, 32, 32, H, b.b3, nullptr, 0)));
    P = b3 + O;
  }
  {
    LossArgs a;
    memset(&a, 0, sizeof(a));
    a.y = L->net[0].y; a.v = L->net[1].y; a.actions = actions; a.logp_old = logp_old; a.adv = adv; a.ret = ret;
    a.dy = L->net[0].dy; a.dv = L->net[1].dy; a.stats = L->stats; a.R = R; a.R_pad = Rkn[0];
    a.dyt = L->net[0].dyt; a.dvt = L->net[1].dyt; a.ldt = Rp;
    a.out_dim = L->pol.out_dim; a.dist = L->pol.dist;
    a.clip = c->clip; a.vf_coef = c->vf_coef; a.ent_coef = c->ent_coef; a.inv_R = 1.0f / (float)R;
    a.G = G; a.Rv = Rn[1]; a.Rv_pad = Rkn[1]; a.inv_Rv = 1.0f / (float)Rn[1];
    a.policy = nets & 1; a.value = (nets >> 1) & 1;
    a.sel = sel;
    hipLaunchKernelGGL((loss_kernel<E>), grid1(Rkn[0]), dim3(256), 0, s, a);
    if (finish) hipLaunchKernelGGL(stats_reduce_kernel, dim3(1), dim3(64), 0, s, L->stats);
    LTRY(hipGetLastError());
  }
  size_t off = 0;
  Reducer red;
  const int64_t ps = L->part_stride;
  for (int n = 0; n < 2; ++n) {
    NetBufs& b = L->net[n];
    const int O = n == 0 ? L->pol.out_dim : 1;
    const int D = Dn[n], Dp = Dpn[n];
    const int64_t R = Rn[n], Rk = Rkn[n];
    const size_t first = (size_t)D * H + H;
    if (!((nets >> n) & 1)) {
      off += net_count(D, H, O, NL);
      continue;
    }
    // offsets into the parameter vector; the kernels write the slices' copies at L->part + offset
    const size_t oW3 = off + first + (size_t)(NL - 1) * mid, ob3 = oW3 + (size_t)H * O;
    auto oW = [&](int l) { return l == 0 ? off : off + first + (size_t)(l - 1) * mid; };          // weights of hidden layer l
    auto ob = [&](int l) { return l == 0 ? off + (size_t)D * H : oW(l) + (size_t)H * H; };       // ... its bias
    float* const part = L->part;
    int used = 0;
    // backward through the activations: dZ of every hidden layer leaves unit-major, its column sums
    // are the bias gradient; the first layer's is not needed row-major
    LTRY((rowgemm<BF16, E, EPI_DTANH>(s, b.dy, Rp, 32, b.wn3, H, 32, NL > 1 ? b.dz[NL - 1] : nullptr, R, H, H, 32, nullptr,
                                      b.h[NL - 1], H, b.dzt[NL - 1], Rp, Rk, part + ob(NL - 1), ps, &used)));
    red.add(ob(NL - 1), H, used);
    for (int l = NL - 2; l >= 0; --l) {
      LTRY((rowgemm<BF16, E, EPI_DTANH>(s, b.dz[l + 1], Rp, H, b.wn[l + 1], H, H, l > 0 ? b.dz[l] : nullptr, R, H, H, H,
                                        nullptr, b.h[l], H, b.dzt[l], Rp, Rk, part + ob(l), ps, &used)));
      red.add(ob(l), H, used);
    }
    // weight gradients: contraction over the rows, split over workgroups; every slice writes a copy of its own
    // (at least 256 rows per slice, and no more slices than fill the chip about once)
    int slices = (int)fmax(1.0, fmin(256.0, (double)(Rk / 256)));
    if (slices > L->part_slices) slices = L->part_slices;
    if (H <= 256) {
      LTRY((wgrad<BF16>(s, b.ht[NL - 1], H, Rp, b.dyt, 32, Rp, part + oW3, H, O, O, Rk, slices, ps, &used)));
      red.add(oW3, (size_t)H * O, used);
      for (int l = NL - 1; l >= 1; --l) {
        LTRY((wgrad<BF16>(s, b.ht[l - 1], H, Rp, b.dzt[l], H, Rp, part + oW(l), H, H, H, Rk, slices, ps, &used)));
        red.add(oW(l), (size_t)H * H, used);
      }
      // (more input units than the kernel's panel holds - the joint observation - go in panels of 256: the same
      // slices of the rows for each, so one reduce job covers the whole tensor)
      for (int d0 = 0; d0 < D; d0 += 256) {
        const int dm = D - d0 < 256 ? D - d0 : 256;
        LTRY((wgrad<BF16>(s, (const E*)xtn[n] + (size_t)d0 * Rp, Dp - d0, Rp, b.dzt[0], H, Rp,
                          part + oW(0) + (size_t)d0 * H, dm, H, H, Rk, slices, ps, &used)));
      }
      red.add(oW(0), (size_t)D * H, used);
    } else {
      LTRY((gemm<BF16, float, EPI_PARTIAL>(s, b.ht[NL - 1], H, Rp, b.dyt, 32, Rp, part + oW3, H, O, O, Rk, nullptr, nullptr, 0, slices, ps, &used)));
      red.add(oW3, (size_t)H * O, used);
      for (int l = NL - 1; l >= 1; --l) {
        LTRY((gemm<BF16, float, EPI_PARTIAL>(s, b.ht[l - 1], H, Rp, b.dzt[l], H, Rp, part + oW(l), H, H, H, Rk, nullptr, nullptr, 0, slices, ps, &used)));
        red.add(oW(l), (size_t)H * H, used);
      }
      LTRY((gemm<BF16, float, EPI_PARTIAL>(s, xtn[n], Dp, Rp, b.dzt[0], H, Rp, part + oW(0), D, H, H, Rk, nullptr, nullptr, 0, slices, ps, &used)));
      red.add(oW(0), (size_t)D * H, used);
    }
    {
      int64_t per_slice = 2048;
      if ((R + per_slice - 1) / per_slice > L->part_slices) per_slice = (R + L->part_slices - 1) / L->part_slices;
      const unsigned ns = (unsigned)((R + per_slice - 1) / per_slice);
      hipLaunchKernelGGL((rowsum_kernel<E>), dim3((unsigned)O, ns), dim3(256), 0, s, (const E*)b.dyt, (int64_t)O, R, Rp,
                         per_slice, part + ob3, ps);
      red.add(ob3, O, (int)ns);
    }
    LTRY(hipGetLastError());
    off += net_count(D, H, O, NL);
  }
  LTRY(red.launch(L, grad, adam, nullptr, s));
  return MSRL_OK;
}

static_assert(ROWS_STAT_BINS == STAT_BINS, "the row kernel and the loss kernel share the bins");

// The same gradient with the activations kept on chip: weights packed into MFMA tiles, one row
// kernel launch per network (forward, loss, backward through the activations; writes the tiled
// unit-major operands), then the weight and bias gradients from those.
int fused_grad_pass(msrl_learner* L, const float* params, int64_t R, const RowSel& sel, const float* obs,
                    const void* actions, const float* logp_old, const float* adv, const float* ret,
                    const msrl_ppo_cfg* c, float* grad, hipStream_t s, const AdamArgs* adam, int nets = 3,
                    bool clear = true, bool finish = true) {
  // nets: bit n set = network n is handled here (1: the policy network only; the value network's pass
  // through device memory writes its own part of grad and adds to the same statistics bins).  clear /
  // finish: zero the bins first / add the bins up at the end
  const int D = L->pol.in_dim, H = L->pol.hidden, kt1 = L->kt1;
  const NetLayout& ly = L->fly;
  const float* b3p[2];
  {
    LearnPackJobs jobs;
    memset(&jobs, 0, sizeof(jobs));
    if (clear) {  // the statistics bins are zeroed on the way
      jobs.clear = L->stats;
      jobs.n_clear = 8 + 5 * STAT_BINS;
    }
    const float* P = params;
    int max_items = 0;
    for (int n = 0; n < 2; ++n) {
      if (!((nets >> n) & 1)) continue;  // (only ever the value network, the last one: P needs no advance)
      const int O = n == 0 ? L->pol.out_dim : 1;
      const float* W1 = P;
      const float* b1 = W1 + (size_t)D * H;
      const float* W2 = b1 + H;
      const float* b2 = W2 + (size_t)H * H;
      const float* W3 = b2 + H;
      b3p[n] = W3 + (size_t)H * O;
      uint8_t* fwd = L->fpacked + (size_t)n * 2 * ly.bytes;
      uint8_t* bwd = fwd + ly.bytes;
      auto job = [&](const float* src, const float* bias, uint8_t* dst, int n_in, int n_out, int64_t s_in,
                     int64_t s_out, int bias_index, int nuc, int kt, int group, int stride, int slot, int linear) {
        LearnPackJob& j = jobs.job[jobs.n++];
        j.src = src; j.bias = bias; j.dst = (u32x4*)dst; j.n_in = n_in; j.n_out = n_out; j.s_in = s_in; j.s_out = s_out;
        j.bias_index = bias_index; j.nuc = nuc; j.kt = kt; j.group = group; j.chunk_stride = stride; j.slot_base = slot;
        j.linear = linear;
        if (nuc * kt * 64 > max_items) max_items = nuc * kt * 64;
      };
      // forward image: layer 1 (bias parts at inputs D, D + 1), chunk blocks of layer 2 (+ bias tile), layer 3
      // next to the chunk it consumes and once more in the block after it
      job(W1, b1, fwd + ly.w1, D, H, H, 1, D, ly.nuc, ly.kt1, ly.kt1, ly.kt1, 0, 1);
      job(W2, b2, fwd + ly.chunks, H, H, H, 1, H, ly.nuc, ly.kt2 + 1, ly.kt2 + 1, ly.chunk_tiles, 0, 0);
      job(W3, nullptr, fwd + ly.chunks, H, O, O, 1, 0, 1, ly.kt2, ly.tpc, ly.chunk_tiles, ly.kt2 + 1 + ly.tpc, 0);
      if (ly.nuc > 1)
        job(W3, nullptr, fwd + ly.chunks + ly.chunk_bytes, H, O, O, 1, 0, 1, ly.kt2 - ly.tpc, ly.tpc, ly.chunk_tiles,
            ly.kt2 + 1, 0);
      // backward image: W3 with the layer-2 units as tile rows (in the layer-1 area), W2 with the layer-1
      // units as tile rows (chunk blocks)
      job(W3, nullptr, bwd + ly.w1, O, H, 1, O, 0, ly.nuc, 1, 1, 1, 0, 0);
      job(W2, nullptr, bwd + ly.chunks, H, H, 1, H, 0, ly.nuc, ly.kt2, ly.kt2, ly.chunk_tiles, 0, 0);
      P = b3p[n] + O;
    }
    hipLaunchKernelGGL(learn_pack_kernel, dim3((unsigned)((max_items + 255) / 256), (unsigned)jobs.n), dim3(256), 0, s,
                       jobs);
    LTRY(hipGetLastError());
  }
  const int64_t n_tiles = (R + 31) / 32;
  const int64_t groups = (n_tiles + rows_waves(H) - 1) / rows_waves(H);
  const int64_t resident = (int64_t)L->cus * rows_workgroups_per_cu(H);
  unsigned grid = (unsigned)(groups < resident ? groups : resident);
  if (H <= 64 && grid > (unsigned)L->part_slices) grid = (unsigned)L->part_slices;  // one copy of the gradient per workgroup
  // 64-unit networks: the row kernel forms the weight gradients itself, one copy per workgroup
  const bool small = H <= 64;
  Reducer red;
  size_t off = 0;
  for (int n = 0; n < 2; ++n) {
    const int O = n == 0 ? L->pol.out_dim : 1;
    const size_t oW1 = off, ob1 = oW1 + (size_t)D * H, oW2 = ob1 + H, ob2 = oW2 + (size_t)H * H, oW3 = ob2 + H,
                 ob3 = oW3 + (size_t)H * O;
    off += net_count(D, H, O);
    if (!((nets >> n) & 1)) continue;
    NetBufs& b = L->net[n];
    RowsArgs a;
    memset(&a, 0, sizeof(a));
    if (small) {
      a.part = L->part; a.part_stride = L->part_stride;
      a.oW1 = (int32_t)oW1; a.ob1 = (int32_t)ob1; a.oW2 = (int32_t)oW2; a.ob2 = (int32_t)ob2; a.oW3 = (int32_t)oW3;
      a.ob3 = (int32_t)ob3;
      const size_t offs[6] = {oW1, ob1, oW2, ob2, oW3, ob3};
      const size_t counts[6] = {(size_t)D * H, (size_t)H, (size_t)H * H, (size_t)H, (size_t)H * O, (size_t)O};
      for (int q = 0; q < 6; ++q) red.add(offs[q], counts[q], (int)grid);
    }
    a.packed = L->fpacked + (size_t)n * 2 * ly.bytes;
    a.b3 = b3p[n];
    a.obs = obs; a.actions = actions; a.logp_old = logp_old; a.adv = adv; a.ret = ret;
    a.R = R; a.n_tiles = n_tiles; a.D = D; a.out_dim = L->pol.out_dim;
    a.obs_vec4 = (D % 4 == 0 && ((uintptr_t)obs & 15) == 0) ? 1 : 0;
    a.sel = sel;
    a.clip = c->clip; a.vf_coef = c->vf_coef; a.ent_coef = c->ent_coef; a.inv_R = 1.0f / (float)R;
    a.xt = (__bf16*)L->xt; a.h1t = (__bf16*)b.ht[0]; a.h2t = (__bf16*)b.ht[1]; a.dz2t = (__bf16*)b.dzt[1];
    a.dz1t = (__bf16*)b.dzt[0]; a.dyt = (__bf16*)b.dyt;
    a.stats = L->stats;
    hipError_t e = H == 64 ? launch_ppo_rows_h64(kt1, n, a, grid, s)
                 : H == 128 ? launch_ppo_rows_h128(kt1, n, a, grid, s)
                            : launch_ppo_rows_h256(kt1, n, a, grid, s);
    LTRY(e);
  }
  LTRY(hipGetLastError());
  if (small) {
    LTRY(red.launch(L, grad, adam, finish ? L->stats : nullptr, s));
    return MSRL_OK;
  }
  off = 0;
  // Slices of row tiles: two compute units' share per slice, i.e. half as many workgroups per contraction as
  // compute units (the six contractions of a pass run two launches deep, so the chip stays busy).  Every
  // slice stores a copy of its result; the copies are added up in slice order afterwards.
  int tps = (int)((n_tiles + L->cus - 1) / L->cus);
  tps = (tps + 1) / 2 * 2 * 2;
  while ((n_tiles + tps - 1) / tps > L->part_slices) tps *= 2;
  const unsigned slices = (unsigned)((n_tiles + tps - 1) / tps);
  // the contractions of both networks in two launches: the four with a hidden layer's width of columns,
  // and the two of the output layers
  WgradTJobs wide, narrow;
  wide.n = narrow.n = 0;
  for (int n = 0; n < 2; ++n) {
    if (!((nets >> n) & 1)) continue;  // (the value network, behind the policy network's gradient)
    NetBufs& b = L->net[n];
    const int O = n == 0 ? L->pol.out_dim : 1;
    const size_t oW1 = off, ob1 = oW1 + (size_t)D * H, oW2 = ob1 + H, ob2 = oW2 + (size_t)H * H, oW3 = ob2 + H,
                 ob3 = oW3 + (size_t)H * O;
    auto wg = [&](const void* A, int UA, int M, const void* B, int UB, int N, size_t oC, int64_t ldc, size_t obias) {
      WgradTArgs& g = N <= 32 ? narrow.job[narrow.n++] : wide.job[wide.n++];
      memset(&g, 0, sizeof(g));
      g.A = (const __bf16*)A; g.B = (const __bf16*)B; g.UA = UA; g.UB = UB; g.M = M; g.N = N; g.m_out = M;
      g.n_tiles = n_tiles; g.tiles_per_slice = tps; g.C = L->part + oC; g.ldc = ldc; g.bias = L->part + obias;
      g.slice_stride = L->part_stride;
      red.add(oC, (size_t)M * ldc, (int)slices);
      red.add(obias, (size_t)N, (int)slices);
    };
    wg(b.ht[1], H, H, b.dyt, 16, O, oW3, O, ob3);
    wg(b.ht[0], H, H, b.dzt[1], H, H, oW2, H, ob2);
    wg(L->xt, 16 * kt1, D, b.dzt[0], H, H, oW1, H, ob1);
    off += net_count(D, H, O);
  }
  if (wide.n)
    hipLaunchKernelGGL((wgrad_tiled_kernel<8, 2>), dim3(slices, (unsigned)wide.n), dim3(512), 0, s, wide);
  if (narrow.n) hipLaunchKernelGGL((wgrad_tiled_kernel<1, 4>), dim3(slices, (unsigned)narrow.n), dim3(512), 0, s, narrow);
  LTRY(hipGetLastError());
  LTRY(red.launch(L, grad, adam, finish ? L->stats : nullptr, s));  // (the bins are complete: the row kernels ran)
  return MSRL_OK;
}

int check_learner_args(const char* who, msrl_learner* L, const void* params, int64_t R, const void* obs,
                       const void* actions, const void* logp_old, const void* adv, const void* ret,
                       const msrl_row_select* rows, const msrl_ppo_cfg* c) {
  if (!L || !params || !obs || !actions || !logp_old || !adv || !ret || !c)
    return fail(MSRL_EINVAL, "%s: NULL argument", who);
  if (R < 1 || R > L->max_rows)
    return fail(MSRL_EINVAL, "%s: %lld rows, the learner was created for 1..%lld", who, (long long)R,
                (long long)L->max_rows);
  if (!(c->clip >= 0.0f)) return fail(MSRL_EINVAL, "%s: clip must be >= 0", who);
  if (R % L->G != 0)
    return fail(MSRL_EINVAL, "%s: %lld rows are no whole groups of %d (the agents of an env, centralised critic)", who,
                (long long)R, L->G);
  if (rows) {
    if (rows->group < 1 || rows->first < 0 || rows->count < 1 || rows->first + rows->count > rows->group)
      return fail(MSRL_EINVAL, "%s: row selection (group %d, first %d, count %d) must satisfy 0 <= first, 1 <= count, "
                               "first + count <= group", who, rows->group, rows->first, rows->count);
    if (L->G > 1)
      return fail(MSRL_EINVAL, "%s: a centralised critic reads whole groups of rows; a row selection is not supported", who);
  }
  return MSRL_OK;
}

AdamArgs adam_args(float* params, float* m, float* v, int64_t k, const msrl_ppo_cfg* cfg) {
  AdamArgs a;
  a.p = params; a.m = m; a.v = v;
  a.lr = cfg->lr; a.b1 = cfg->beta1; a.b2 = cfg->beta2; a.eps = cfg->adam_eps;
  a.c1 = (float)(1.0 - pow((double)cfg->beta1, (double)k));
  a.c2 = (float)(1.0 - pow((double)cfg->beta2, (double)k));
  return a;
}

RowSel selection(const msrl_row_select* rows, int64_t row0) {
  return rows ? RowSel{row0, rows->group, rows->first, rows->count} : RowSel{row0, 0, 0, 0};
}

// the gradient of logical rows [row0, row0 + R) of the selection, into grad; with `adam`, the Adam step on
// every element follows inside the kernel that finishes the gradient
int grad_rows(msrl_learner* L, const float* params, int64_t R, int64_t row0, const msrl_row_select* rows,
              const float* obs, const void* actions, const float* logp_old, const float* adv, const float* ret,
              const msrl_ppo_cfg* cfg, float* grad, hipStream_t s, const AdamArgs* adam = nullptr) {
  const RowSel sel = selection(rows, row0);
  if (L->fused) return fused_grad_pass(L, params, R, sel, obs, actions, logp_old, adv, ret, cfg, grad, s, adam);
  if (L->fused_policy) {
    // Centralised critic: the policy network on chip, then the value network (one row per group, a wide
    // first layer) through device memory; it adds its part of grad and of the statistics.  (Running the
    // second pass on a stream of its own beside the first was measured: no gain, the row kernel's
    // workgroups leave no LDS for the value network's kernels to start beside them.)
    // (With an Adam step folded in, each pass steps its own network's parameters: the value network's pass reads
    // none of the policy network's.)
    int rc = fused_grad_pass(L, params, R, sel, obs, actions, logp_old, adv, ret, cfg, grad, s, adam, 1, true, false);
    if (rc == MSRL_OK) rc = grad_pass<true>(L, params, R, sel, obs, actions, logp_old, adv, ret, cfg, grad, s, adam, 2, true);
    return rc;
  }
  return L->bf16 ? grad_pass<true>(L, params, R, sel, obs, actions, logp_old, adv, ret, cfg, grad, s, adam)
                 : grad_pass<false>(L, params, R, sel, obs, actions, logp_old, adv, ret, cfg, grad, s, adam);
}

}  // namespace

extern "C" {

int msrl_learner_init(const msrl_policy_cfg* policy, int64_t max_rows, msrl_learner** out) {
  return msrl_learner_init_path(policy, max_rows, MSRL_LEARNER_PATH_AUTO, out);
}

int msrl_learner_init_path(const msrl_policy_cfg* policy, int64_t max_rows, int32_t path, msrl_learner** out) {
  if (!policy || !out) return fail(MSRL_EINVAL, "msrl_learner_init: NULL argument");
  if (path != MSRL_LEARNER_PATH_AUTO && path != MSRL_LEARNER_PATH_DEVICE_MEMORY)
    return fail(MSRL_EINVAL, "msrl_learner_init_path: unknown path %d", path);
  *out = nullptr;
  if (policy->in_dim < 1 || policy->hidden < 32 || policy->hidden % 32 != 0 || policy->out_dim < 1 ||
      policy->out_dim > 32 || (policy->dtype != MSRL_F32 && policy->dtype != MSRL_BF16) ||
      (policy->dist != MSRL_CATEGORICAL && policy->dist != MSRL_DIAG_GAUSSIAN) ||
      (policy->dist == MSRL_DIAG_GAUSSIAN && policy->out_dim % 2 != 0))
    return fail(MSRL_EINVAL, "msrl_learner_init: unsupported policy configuration (hidden must be a multiple of "
                             "32, out_dim at most 32)");
  if (policy->hidden_layers != 0 && (policy->hidden_layers < 2 || policy->hidden_layers > MAX_LAYERS))
    return fail(MSRL_EINVAL, "msrl_learner_init: hidden_layers must be 0 (two) or 2..8");
  if (policy->roles > 1)
    return fail(MSRL_EINVAL, "msrl_learner_init: a learner holds one parameter set; create one per role");
  if (policy->value_in_dim < 0 || (policy->value_in_dim != 0 && policy->value_in_dim % policy->in_dim != 0))
    return fail(MSRL_EINVAL, "msrl_learner_init: value_in_dim %d is no multiple of in_dim %d", policy->value_in_dim,
                policy->in_dim);
  if (max_rows < 1) return fail(MSRL_EINVAL, "msrl_learner_init: max_rows must be positive");
  msrl_learner* L = new (std::nothrow) msrl_learner;
  if (!L) return fail(MSRL_ENOMEM, "msrl_learner_init: host allocation failed");
  memset(L, 0, sizeof(*L));
  L->pol = *policy;
  L->max_rows = max_rows;
  L->Rp = round_up(max_rows, 128);
  L->Dp = (int)round_up(policy->in_dim, 16);
  L->bf16 = policy->dtype == MSRL_BF16;
  L->esz = L->bf16 ? 2 : 4;
  L->layers = policy->hidden_layers == 0 ? 2 : policy->hidden_layers;
  L->G = policy->value_in_dim > policy->in_dim ? policy->value_in_dim / policy->in_dim : 1;
  L->Dvp = (int)round_up((int64_t)L->G * policy->in_dim, 16);
  L->n_params = net_count(policy->in_dim, policy->hidden, policy->out_dim, L->layers) +
                net_count(L->G * policy->in_dim, policy->hidden, 1, L->layers);
  const size_t H = (size_t)policy->hidden, Rp = (size_t)L->Rp, Dp = (size_t)L->Dp, e = L->esz;
  L->kt1 = policy->in_dim + 2 <= 32 ? 2 : 4;
  L->fused_policy = L->bf16 && policy->dist == MSRL_CATEGORICAL && policy->out_dim <= 16 && policy->in_dim + 2 <= 64 &&
                    (policy->hidden == 64 || policy->hidden == 128 || policy->hidden == 256) && L->layers == 2 &&
                    path != MSRL_LEARNER_PATH_DEVICE_MEMORY;
  L->fused = L->fused_policy && L->G == 1;
  L->fly = net_layout(16 * L->kt1 - 1, policy->hidden, true);
  int rc = MSRL_OK;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
      delete L;
      return fail(MSRL_EDEVICE, "msrl_learner_init: cannot query the device");
    }
    L->cus = cus;
  }
  auto A = [&](void** p, size_t bytes) { if (rc == MSRL_OK) rc = dev_alloc((uint8_t**)p, bytes); };
  A(&L->xc, Rp * Dp * e);
  A(&L->xt, (L->fused_policy && (size_t)(16 * L->kt1) > Dp ? (size_t)(16 * L->kt1) : Dp) * Rp * e);
  if (L->fused_policy) A((void**)&L->fpacked, 4 * L->fly.bytes);
  if (L->G > 1) {
    A(&L->xcv, (Rp / L->G + 128) * (size_t)L->Dvp * e);
    A(&L->xtv, (size_t)L->Dvp * Rp * e);
  }
  for (int n = 0; n < 2; ++n) {
    NetBufs& b = L->net[n];
    for (int l = 0; l < L->layers; ++l) {
      A(&b.wt[l], H * (l == 0 ? (n == 1 && L->G > 1 ? (size_t)L->Dvp : Dp) : H) * e);
      if (l >= 1) A(&b.wn[l], H * H * e);
      A(&b.h[l], Rp * H * e);
      A(&b.ht[l], H * Rp * e);
      if (l >= 1) A(&b.dz[l], Rp * H * e);
      A(&b.dzt[l], H * Rp * e);
    }
    A(&b.wt3, 32 * H * e);
    A(&b.wn3, H * 32 * e);
    A((void**)&b.b3, 32 * sizeof(float));
    A((void**)&b.y, Rp * 32 * sizeof(float));
    A(&b.dy, Rp * 32 * e);
    A(&b.dyt, 32 * Rp * e);
  }
  A((void**)&L->grad, L->n_params * sizeof(float));
  // a contraction over the rows is split into at most this many slices (never more than one per 128 rows)
  L->part_slices = (int)(L->Rp / 128 + 1 < 256 ? L->Rp / 128 + 1 : 256);
  L->part_stride = round_up((int64_t)L->n_params, 64);
  A((void**)&L->part, (size_t)L->part_slices * (size_t)L->part_stride * sizeof(float));
  A((void**)&L->stats, (8 + 5 * STAT_BINS) * sizeof(float));
  if (rc != MSRL_OK) {
    msrl_learner_destroy(L);
    return rc;
  }
  *out = L;
  return MSRL_OK;
}

void msrl_learner_destroy(msrl_learner* L) {
  if (!L) return;
  void* ptrs[] = {L->xc, L->xt, L->xcv, L->xtv, L->grad, L->part, L->stats, L->fpacked};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  for (int n = 0; n < 2; ++n) {
    NetBufs& b = L->net[n];
    void* q[] = {b.wt3, b.wn3, b.b3, b.y, b.dy, b.dyt};
    for (void* p : q)
      if (p) (void)hipFree(p);
    for (int l = 0; l < MAX_LAYERS; ++l) {
      void* r[] = {b.wt[l], b.wn[l], b.h[l], b.ht[l], b.dz[l], b.dzt[l]};
      for (void* p : r)
        if (p) (void)hipFree(p);
    }
  }
  delete L;
}

int msrl_ppo_grad(msrl_learner* L, const float* params, int64_t R, const float* obs, const void* actions,
                  const float* logp_old, const float* adv, const float* ret, const msrl_row_select* rows,
                  const msrl_ppo_cfg* cfg, float* grad, float* stats, void* hip_stream) {
  int rc = check_learner_args("msrl_ppo_grad", L, params, R, obs, actions, logp_old, adv, ret, rows, cfg);
  if (rc != MSRL_OK) return rc;
  if (!grad) return fail(MSRL_EINVAL, "msrl_ppo_grad: grad is NULL");
  hipStream_t s = (hipStream_t)hip_stream;
  rc = grad_rows(L, params, R, 0, rows, obs, actions, logp_old, adv, ret, cfg, grad, s);
  if (rc != MSRL_OK) return rc;
  if (stats) LTRY(hipMemcpyAsync(stats, L->stats, 5 * sizeof(float), hipMemcpyDeviceToDevice, s));
  return MSRL_OK;
}

int msrl_rows_mean(const float* x, int64_t R, const msrl_row_select* rows, float* out, void* hip_stream) {
  if (!x || !out) return fail(MSRL_EINVAL, "msrl_rows_mean: NULL argument");
  if (R < 1) return fail(MSRL_EINVAL, "msrl_rows_mean: R must be positive");
  if (rows && (rows->group < 1 || rows->first < 0 || rows->count < 1 || rows->first + rows->count > rows->group))
    return fail(MSRL_EINVAL, "msrl_rows_mean: bad row selection");
  hipStream_t s = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(64), 0, s, out, (int64_t)1, 0.0f);
  const int64_t blocks = (R + 256 * 16 - 1) / (256 * 16);
  hipLaunchKernelGGL(rows_sum_kernel, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0, s, x,
                     selection(rows, 0), R, 1.0f / (float)R, out);
  LTRY(hipGetLastError());
  return MSRL_OK;
}

int msrl_adam_step(float* params, float* m, float* v, const float* grad, int64_t n, int64_t k,
                   const msrl_ppo_cfg* cfg, void* hip_stream) {
  if (!params || !m || !v || !grad || !cfg) return fail(MSRL_EINVAL, "msrl_adam_step: NULL argument");
  if (n < 0 || k < 1) return fail(MSRL_EINVAL, "msrl_adam_step: n must be >= 0 and the step counter >= 1");
  if (n == 0) return MSRL_OK;
  const AdamArgs a = adam_args(params, m, v, k, cfg);
  hipLaunchKernelGGL(adam_kernel, grid1(n), dim3(256), 0, (hipStream_t)hip_stream, a, grad, n);
  LTRY(hipGetLastError());
  return MSRL_OK;
}

int msrl_params_cast(const float* master, void* out, int64_t n, int32_t dtype, void* hip_stream) {
  if (!master || !out) return fail(MSRL_EINVAL, "msrl_params_cast: NULL argument");
  if (n < 0 || (dtype != MSRL_F32 && dtype != MSRL_BF16)) return fail(MSRL_EINVAL, "msrl_params_cast: bad size or dtype");
  if (n == 0) return MSRL_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == MSRL_BF16)
    LTRY(convert_pad(s, master, 1, n, n, (__bf16*)out, n, 1));
  else
    LTRY(convert_pad(s, master, 1, n, n, (float*)out, n, 1));
  return MSRL_OK;
}

int msrl_ppo_update(msrl_learner* L, float* params, float* m, float* v, int64_t* step_counter, int64_t R,
                    int32_t iters, int32_t minibatches, const float* obs, const void* actions,
                    const float* logp_old, const float* adv, const float* ret, const msrl_row_select* rows,
                    const msrl_ppo_cfg* cfg, void* hip_stream) {
  if (!L || !params || !m || !v || !step_counter || !obs || !actions || !logp_old || !adv || !ret || !cfg)
    return fail(MSRL_EINVAL, "msrl_ppo_update: NULL argument");
  if (iters < 1 || minibatches < 1 || R < minibatches)
    return fail(MSRL_EINVAL, "msrl_ppo_update: iters and minibatches must be positive and R >= minibatches");
  if (R % L->G != 0 || R / L->G < minibatches)
    return fail(MSRL_EINVAL, "msrl_ppo_update: %lld rows are no whole groups of %d, or fewer groups than minibatches",
                (long long)R, L->G);
  const int64_t block = R / minibatches / L->G * L->G;  // whole groups (the agents of an env) per block
  const int64_t largest = R - block * (minibatches - 1);
  if (largest > L->max_rows)
    return fail(MSRL_EINVAL, "msrl_ppo_update: a minibatch of %lld rows exceeds the learner's %lld",
                (long long)largest, (long long)L->max_rows);
  int rc = check_learner_args("msrl_ppo_update", L, params, largest, obs, actions, logp_old, adv, ret, rows, cfg);
  if (rc != MSRL_OK) return rc;
  for (int it = 0; it < iters; ++it)
    for (int b = 0; b < minibatches; ++b) {
      const int64_t r0 = (int64_t)b * block, r1 = b == minibatches - 1 ? R : r0 + block;
      // the Adam step rides on the kernel that adds up the slices of the gradient
      *step_counter += 1;
      const AdamArgs adam = adam_args(params, m, v, *step_counter, cfg);
      rc = grad_rows(L, params, r1 - r0, r0, rows, obs, actions, logp_old, adv, ret, cfg, L->grad,
                     (hipStream_t)hip_stream, &adam);
      if (rc != MSRL_OK) {
        *step_counter -= 1;  // nothing was enqueued for this step
        return rc;
      }
    }
  return MSRL_OK;
}

}  // extern "C"
