// n4  SliM-LLM+ on one linear layer (Sec. 3.4; Sec. 4; App. B): the widths of SBA stay, SQC and the error compensation
// are left out, and every (row, group) gets a quantiser with learnable weight clipping whose two clipping strengths
// are trained with AdamW on the layer-output error.  The paper names the method it borrows (the learnable weight
// clipping of OmniQuant) and the optimiser; the forward pass built here is
//     hi = sigmoid(gamma) max_j w_j,  lo = sigmoid(beta) min_j w_j,  delta = (hi - lo) / (2^b - 1),
//     z = -round(lo / delta),  q_j = clamp(round(w_j / delta) + z, 0, 2^b - 1),  w_hat_j = delta (q_j - z)
// (Eq. 1 on the clipped range, every width in this affine form), the loss L = tr(dW G dW^T) / (n T), the mean
// squared error of the layer's outputs over the T calibration tokens (Eq. 3), taken full batch: it depends on X only
// through G = X X^T, so one step sees all tokens.  The backward pass takes the rounding as the identity and lets the
// clamp pass derivatives where it does not clip:
//     g = dL/dW_hat = 2 (W_hat - W) G / (n T)                                (fp64 matrix cores)
//     dW_hat_j / d delta = (q_j - z) - w_j / delta   or, clipped,   (q_j - z) - lo / delta
//     dW_hat_j / d lo at fixed delta = 0   or, clipped,   1
// Everything is fp64; one wavefront per (row, group) in both elementwise kernels, fixed-order reductions.
#include <cmath>

#include "slim_device.h"
#include "slim_internal.h"

namespace {

using namespace slimdev;

struct LwcGroup {
  double M, m_, s_hi, s_lo, lo, delta, z, Q;
  bool live;
};

// parameters of one (row, group) from its extreme values and clipping strengths; wavefront-uniform
__device__ __forceinline__ LwcGroup lwc_group(double M, double m_, double gamma, double betap, int bits) {
  LwcGroup p;
  p.M = M;
  p.m_ = m_;
  p.Q = (double)((1 << bits) - 1);
  p.s_hi = 1.0 / (1.0 + exp(-gamma));
  p.s_lo = 1.0 / (1.0 + exp(-betap));
  const double hi = p.s_hi * M;
  p.lo = p.s_lo * m_;
  p.live = hi > p.lo;
  p.delta = p.live ? (hi - p.lo) / p.Q : 1.0;
  p.z = p.live ? -rint(p.lo / p.delta) : 0.0;
  return p;
}

struct LwcArgs {
  const double* W;        // n x m fp64 (ld = m)
  int n, m, beta;
  const uint8_t* bits;    // k
  double* gamma;          // n x k each
  double* betap;
  double* m1g;
  double* vg;
  double* m1b;
  double* vb;
  double* D;              // n x m: W_hat - W
  const double* DG;       // n x m: D G
  double* lp;             // n x k: sum_j D_j DG_j of the (row, group)
  double gscale;          // 2 / (n T)
  double lr, b1, b2, eps, c1, c2;   // AdamW; c1 = 1 - b1^step, c2 = 1 - b2^step
  // final quantisation
  uint8_t* codes;         // n x m (ld = m)
  double* scale;          // n x k
  double* zero;
  void* What;
  int what_f64;
};

__device__ __forceinline__ void lwc_extremes(const double* w, int beta, int lane, double& M, double& m_) {
  double mx = -INFINITY, mn = INFINITY;
  for (int c = lane; c < beta; c += 64) {
    const double v = w[c];
    mx = fmax(mx, v);
    mn = fmin(mn, v);
  }
  M = wave_max(mx);
  m_ = wave_min(mn);
}

// MODE 0: D = W_hat - W.   MODE 1: the final quantisation (codes, scale, zero, W_hat).
template <int MODE>
__global__ __launch_bounds__(256) void lwc_forward_kernel(LwcArgs a) {
  const int lane = threadIdx.x & 63;
  const int k = a.m / a.beta;
  const int64_t unit = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= (int64_t)a.n * k) return;
  const int row = (int)(unit / k), g = (int)(unit % k);
  const int64_t base = (int64_t)row * a.m + (int64_t)g * a.beta;
  const double* w = a.W + base;
  double M, m_;
  lwc_extremes(w, a.beta, lane, M, m_);
  const int bits = min(max((int)a.bits[g], 1), 8);
  const LwcGroup p = lwc_group(M, m_, a.gamma[unit], a.betap[unit], bits);
  for (int c = lane; c < a.beta; c += 64) {
    const double wv = w[c];
    const double q = fmin(fmax(rint(wv / p.delta) + p.z, 0.0), p.Q);
    const double what = p.delta * (q - p.z);
    if (MODE == 0) {
      a.D[base + c] = what - wv;
    } else {
      a.codes[base + c] = (uint8_t)q;
      if (a.What) {
        if (a.what_f64)
          static_cast<double*>(a.What)[base + c] = what;
        else
          static_cast<float*>(a.What)[base + c] = (float)what;
      }
    }
  }
  if (MODE == 1 && lane == 0) {
    a.scale[unit] = p.delta;
    a.zero[unit] = p.z;
  }
}

// derivatives of the (row, group)'s two strengths, their AdamW step, and the (row, group)'s share of the loss
__global__ __launch_bounds__(256) void lwc_backward_adam(LwcArgs a) {
  const int lane = threadIdx.x & 63;
  const int k = a.m / a.beta;
  const int64_t unit = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= (int64_t)a.n * k) return;
  const int row = (int)(unit / k), g = (int)(unit % k);
  const int64_t base = (int64_t)row * a.m + (int64_t)g * a.beta;
  const double* w = a.W + base;
  double M, m_;
  lwc_extremes(w, a.beta, lane, M, m_);
  const int bits = min(max((int)a.bits[g], 1), 8);
  const double gamma = a.gamma[unit], betap = a.betap[unit];
  const LwcGroup p = lwc_group(M, m_, gamma, betap, bits);
  double s1 = 0.0, s2 = 0.0, lsum = 0.0;
  for (int c = lane; c < a.beta; c += 64) {
    const double wv = w[c];
    const double u = rint(wv / p.delta) + p.z;
    const double q = fmin(fmax(u, 0.0), p.Q);
    const bool inside = (u >= 0.0) && (u <= p.Q);
    const double dg = a.DG[base + c];
    const double gj = a.gscale * dg;
    const double dwd = inside ? (q - p.z) - wv / p.delta : (q - p.z) - p.lo / p.delta;
    s1 += gj * dwd;
    s2 += inside ? 0.0 : gj;
    lsum += a.D[base + c] * dg;
  }
  s1 = wave_sum(s1);
  s2 = wave_sum(s2);
  lsum = wave_sum(lsum);
  if (lane != 0) return;
  a.lp[unit] = lsum;
  const double d_hi = p.live ? s1 / p.Q : 0.0;
  const double d_lo = p.live ? -s1 / p.Q + s2 : 0.0;
  const double gg = d_hi * p.M * p.s_hi * (1.0 - p.s_hi);
  const double gb = d_lo * p.m_ * p.s_lo * (1.0 - p.s_lo);
  {
    const double m1 = a.b1 * a.m1g[unit] + (1.0 - a.b1) * gg;
    const double v = a.b2 * a.vg[unit] + (1.0 - a.b2) * gg * gg;
    a.m1g[unit] = m1;
    a.vg[unit] = v;
    a.gamma[unit] = gamma - a.lr * (m1 / a.c1) / (sqrt(v / a.c2) + a.eps);
  }
  {
    const double m1 = a.b1 * a.m1b[unit] + (1.0 - a.b1) * gb;
    const double v = a.b2 * a.vb[unit] + (1.0 - a.b2) * gb * gb;
    a.m1b[unit] = m1;
    a.vb[unit] = v;
    a.betap[unit] = betap - a.lr * (m1 / a.c1) / (sqrt(v / a.c2) + a.eps);
  }
}

// the (row, group)'s share of the loss alone (after the last step)
__global__ __launch_bounds__(256) void lwc_loss_kernel(LwcArgs a) {
  const int lane = threadIdx.x & 63;
  const int k = a.m / a.beta;
  const int64_t unit = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= (int64_t)a.n * k) return;
  const int64_t base = (unit / k) * a.m + (unit % k) * a.beta;
  double lsum = 0.0;
  for (int c = lane; c < a.beta; c += 64) lsum += a.D[base + c] * a.DG[base + c];
  lsum = wave_sum(lsum);
  if (lane == 0) a.lp[unit] = lsum;
}

__global__ __launch_bounds__(256) void lwc_fill(double* p, int64_t n, double v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = v;
}

}  // namespace

size_t slim_ws_need_lwc(int n, int m, int beta, int steps) {
  const size_t nk = (size_t)n * (m / beta);
  return 3 * slim_ws_round(sizeof(double) * (size_t)n * m) + slim_ws_round(sizeof(double) * (size_t)m * m) +
         7 * slim_ws_round(sizeof(double) * nk) + slim_ws_round(sizeof(double) * (size_t)(steps + 1));
}

extern "C" slim_status slim_lwc_quantize(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                                         const float* G, int64_t ldg, int64_t n_tokens, const uint8_t* bits, int beta,
                                         int steps, double lr, double beta1, double beta2, double eps, double init,
                                         uint8_t* codes, double* scale, double* zero, void* What,
                                         slim_dtype what_dtype, double* loss_curve) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, W && G && bits && codes && scale && zero, "slim_lwc_quantize: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "slim_lwc_quantize: need n, m > 0 and beta | m");
  SLIM_REQUIRE(ctx, m % 4 == 0 && ldw >= m && ldw % 4 == 0 && ldg >= m && ldg % 4 == 0,
               "slim_lwc_quantize: m, ldw and ldg must be multiples of 4");
  SLIM_REQUIRE(ctx, slim_aligned16(W) && slim_aligned16(G), "slim_lwc_quantize: misaligned pointer");
  SLIM_REQUIRE(ctx, n_tokens > 0 && steps >= 0 && steps <= 100000, "slim_lwc_quantize: need n_tokens > 0 and 0 <= steps <= 100000");
  SLIM_REQUIRE(ctx, lr > 0.0 && beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0 && eps > 0.0,
               "slim_lwc_quantize: need lr > 0, 0 <= beta1, beta2 < 1, eps > 0");
  if (w_dtype != SLIM_F16 && w_dtype != SLIM_BF16 && w_dtype != SLIM_F32)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_lwc_quantize: W must be F16, BF16 or F32");
  if (What && what_dtype != SLIM_F32 && what_dtype != SLIM_F64)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_lwc_quantize: What must be F32 or F64");
  const int k = m / beta;
  SLIM_REQUIRE(ctx, (size_t)k <= (size_t)SLIM_HPIN_BYTES && sizeof(double) * (size_t)(steps + 1) <= (size_t)SLIM_HPIN_BYTES,
               "slim_lwc_quantize: too many groups or steps for the staging buffer");
  // the widths are validated before anything is written (not a hot path: the host waits for them)
  uint8_t* bits_h = reinterpret_cast<uint8_t*>(ctx->hpin);
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(bits_h, bits, k, hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  for (int g = 0; g < k; ++g)
    SLIM_REQUIRE(ctx, bits_h[g] >= 1 && bits_h[g] <= 8, "slim_lwc_quantize: bits[%d] = %d is outside 1..8", g, (int)bits_h[g]);

  slim_status st = slim_ws_reserve(ctx, slim_ws_need_lwc(n, m, beta, steps));
  if (st != SLIM_OK) return st;
  const size_t nk = (size_t)n * k;
  double* W64 = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)n * m));
  double* D = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)n * m));
  double* DG = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)n * m));
  double* G64 = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)m * m));
  double* par[6];
  for (double*& p : par) p = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * nk));
  double* lp = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * nk));
  double* loss = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)(steps + 1)));

  st = slim_widen_f64(ctx, "lwc_widen_w", W, w_dtype, n, m, ldw, W64, (int64_t)m);
  if (st != SLIM_OK) return st;
  st = slim_widen_f64(ctx, "lwc_widen_g", G, SLIM_F32, m, m, ldg, G64, (int64_t)m);
  if (st != SLIM_OK) return st;
  const int fgrid = (int)std::min<size_t>((nk + 255) / 256, 65536);
  SLIM_LAUNCH(ctx, "lwc_init", lwc_fill, dim3(fgrid), dim3(256), 0, par[0], (int64_t)nk, init);
  SLIM_LAUNCH(ctx, "lwc_init", lwc_fill, dim3(fgrid), dim3(256), 0, par[1], (int64_t)nk, init);
  for (int i = 2; i < 6; ++i) SLIM_LAUNCH(ctx, "lwc_init", lwc_fill, dim3(fgrid), dim3(256), 0, par[i], (int64_t)nk, 0.0);

  LwcArgs a;
  a.W = W64;
  a.n = n;
  a.m = m;
  a.beta = beta;
  a.bits = bits;
  a.gamma = par[0];
  a.betap = par[1];
  a.m1g = par[2];
  a.vg = par[3];
  a.m1b = par[4];
  a.vb = par[5];
  a.D = D;
  a.DG = DG;
  a.lp = lp;
  a.gscale = 2.0 / ((double)n * (double)n_tokens);
  a.lr = lr;
  a.b1 = beta1;
  a.b2 = beta2;
  a.eps = eps;
  a.c1 = a.c2 = 1.0;
  a.codes = codes;
  a.scale = scale;
  a.zero = zero;
  a.What = What;
  a.what_f64 = (what_dtype == SLIM_F64);
  const dim3 grid(slim_cdiv((int64_t)nk, 4)), block(256);
  slim_gemm_desc d;
  d.A = D;
  d.lda = m;
  d.B = G64;
  d.ldb = m;
  d.C = DG;
  d.ldc = m;
  d.C2 = nullptr;
  d.ldc2 = 0;
  d.M = n;
  d.N = m;
  d.K = m;
  d.flags = 0;
  d.alpha = 1.0;
  d.beta = 0.0;
  for (int it = 1; it <= steps + 1; ++it) {
    SLIM_LAUNCH(ctx, "lwc_forward", lwc_forward_kernel<0>, grid, block, 0, a);
    st = slim_dgemm(ctx, "lwc_grad_dgemm", 0, d);
    if (st != SLIM_OK) return st;
    if (it <= steps) {
      a.c1 = 1.0 - std::pow(beta1, (double)it);
      a.c2 = 1.0 - std::pow(beta2, (double)it);
      SLIM_LAUNCH(ctx, "lwc_backward_adam", lwc_backward_adam, grid, block, 0, a);
    } else {
      SLIM_LAUNCH(ctx, "lwc_loss", lwc_loss_kernel, grid, block, 0, a);
    }
    st = slim_sum_f64(ctx, "lwc_loss_sum", lp, (int)nk, loss + (it - 1));
    if (st != SLIM_OK) return st;
  }
  SLIM_LAUNCH(ctx, "lwc_final", lwc_forward_kernel<1>, grid, block, 0, a);
  if (!loss_curve) return SLIM_OK;                 // nothing for the host: the call does not wait
  double* host = reinterpret_cast<double*>(ctx->hpin);
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(host, loss, sizeof(double) * (size_t)(steps + 1), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  const double norm = (double)n * (double)n_tokens;
  for (int i = 0; i <= steps; ++i) loss_curve[i] = host[i] / norm;
  return SLIM_OK;
}
