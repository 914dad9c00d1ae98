// Host-side launchers of the gfx950 kernels.  All tensors are fp32, channels-last on the
// device: activations N,(D,)H,W,C; filters K,(kd,)kh,kw,C ("KRSC") plus a transposed copy
// C,(kd,)kh,kw,K ("CRSK") for the data gradient.  Every launcher checks its operands on
// the host and returns hipErrorInvalidValue instead of launching on a mismatch.
// All kernels are deterministic (fixed-order reductions, no atomics) and do not depend on
// where in memory a tensor sits beyond 256-byte alignment.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pk {

struct ConvGeom {
    int N, C, D, H, W;     // input, channels-last N,D,H,W,C (D == 1 for 2-d)
    int Clive = 0;         // > 0: only the first Clive of the C input channels can be non-zero in x and in the filter (a
                           // network input of one to three channels is stored with zero channels up to four)
    int K;                 // output channels
    int Do, Ho, Wo;        // output spatial size
    int kd, kh, kw, sd, sh, sw, pd, ph, pw;
    int64_t rows_out() const { return (int64_t)N * Do * Ho * Wo; }
    int64_t rows_in() const { return (int64_t)N * D * H * W; }
    int64_t taps() const { return (int64_t)kd * kh * kw; }
};

// y[N,Do,Ho,Wo,K] = cross-correlation of x with w_krsc (implicit GEMM M=rows_out, N=K, K=taps*C).
// bn_tiles (optional, 16-byte aligned, 2 * tiles_m * K floats): the kernel also leaves, per tile of
// consecutive output rows, the per-channel mean [K] and sum of squared deviations from it [K] of that
// tile's rows of y -- the batch-normalisation statistics pass, taken while the results are still on chip.
// Only where conv_fwd_bn_tiles() says so.
// workspace: conv_fwd_workspace(g) bytes (16-byte aligned) when that is not zero -- a GEMM with few tiles and a long
// reduction is split over the reduction into partial results there, summed in a fixed order; such a launch leaves no bn_tiles.
hipError_t conv_fwd(const float *x, const float *w_krsc, float *y, const ConvGeom &g, hipStream_t s, float *bn_tiles = nullptr,
                    float *workspace = nullptr);
size_t conv_fwd_workspace(const ConvGeom &g);
// whether conv_fwd can produce bn_tiles for these operands, and their layout: tile t covers output
// rows [t * rows_per_tile, min(rows_out, (t + 1) * rows_per_tile))
bool conv_fwd_bn_tiles(const float *x, const float *w_krsc, const ConvGeom &g, int *tiles_m, int *rows_per_tile);
// dx[N,D,H,W,C] (+)= data gradient; w_crsk is the transposed filter copy
hipError_t conv_dgrad(const float *dy, const float *w_crsk, float *dx, const ConvGeom &g, bool accumulate, hipStream_t s,
                      float *workspace = nullptr);
size_t conv_dgrad_workspace(const ConvGeom &g);   // bytes conv_dgrad needs at `workspace` (0: none)
// bytes of split-K workspace conv_wgrad needs for this geometry (0 if none)
size_t conv_wgrad_workspace(const ConvGeom &g);
// dw_krsc[K,taps,C] = filter gradient, deterministic split-K through `workspace`
hipError_t conv_wgrad(const float *dy, const float *x, float *dw_krsc, float *workspace, const ConvGeom &g, hipStream_t s);

// names of the kernel variants the three launchers above pick for a geometry
const char *conv_fwd_kernel(const ConvGeom &g, bool bn_tiles = false);
const char *conv_dgrad_kernel(const ConvGeom &g);
const char *conv_wgrad_kernel(const ConvGeom &g);

// running averages a statistics pass also updates (both pointers null: none):
// mean <- decay * mean + (1 - decay) * batch mean, var <- decay * var + (1 - decay) * batch variance * M / max(M - 1, 1)
struct BnRun {
    float *mean = nullptr, *var = nullptr;
    float decay = 0.f;
};
// number of floats of scratch the BN reductions need for an [M][C] tensor
size_t bn_workspace_floats(int64_t M, int C);
// batch statistics (mean, 1/sqrt(var+eps)) then y = gamma*(x-mean)*istd + beta; relu: y = max(y, 0)
hipError_t bn_fwd(const float *x, const float *gamma, const float *beta, float *y, float *mean, float *istd,
                  float *ws, int64_t M, int C, float eps, bool relu, BnRun run, hipStream_t s);
// floats of the buffer conv_fwd's bn_tiles and bn_fwd_from_tiles share (the tiles plus room to fold them)
size_t bn_tiles_workspace_floats(int tiles_m, int C);
// the same from per-tile statistics left by conv_fwd (tiles[t][0][C] = mean, tiles[t][1][C] = sum of squared
// deviations of rows [t * rows_per_tile, ...)): merges them per channel in double, then applies
hipError_t bn_fwd_from_tiles(const float *x, const float *gamma, const float *beta, float *y, float *mean, float *istd,
                             float *tiles, int tiles_m, int rows_per_tile, int64_t M, int C, float eps, bool relu, BnRun run,
                             hipStream_t s);
// the statistics alone (for a normalisation that is applied inside its consumer), from x or from conv_fwd's tiles
hipError_t bn_stats(const float *x, float *mean, float *istd, float *ws, int64_t M, int C, float eps, BnRun run, hipStream_t s);
hipError_t bn_stats_from_tiles(float *tiles, int tiles_m, int rows_per_tile, int64_t M, int C, float eps, float *mean, float *istd,
                               BnRun run, hipStream_t s);
// z = max(bn(x) + other, 0) with given statistics: a residual branch's normalisation inside the add + ReLU;
// with gamma2 ... istd2 (all four or none) the other input is normalised too: z = max(bn(x) + bn2(other), 0)
hipError_t bn_add_relu_fwd(const float *x, const float *other, const float *gamma, const float *beta, const float *mean,
                           const float *istd, const float *gamma2, const float *beta2, const float *mean2, const float *istd2,
                           float *z, int64_t M, int C, hipStream_t s);
// apply only, with saved statistics (used when a BN output is recomputed)
hipError_t bn_apply(const float *x, const float *gamma, const float *beta, const float *mean, const float *istd,
                    float *y, int64_t M, int C, bool relu, hipStream_t s);
// dgamma, dbeta and dx (dx may alias dy; null: dgamma and dbeta only, dy is not touched); accumulate adds into dx
// instead of overwriting.
// relu: dy is the gradient of max(bn(x), 0); the decision bn(x) > 0 is re-derived from x.
hipError_t bn_bwd(const float *x, const float *dy, const float *gamma, const float *beta, const float *mean, const float *istd,
                  float *dx, float *dgamma, float *dbeta, float *ws, int64_t M, int C, bool accumulate, bool relu, hipStream_t s);

hipError_t relu_fwd(const float *x, float *y, int64_t n, hipStream_t s);
// dx (+)= dy where y > 0 (dx may alias dy when not accumulating)
hipError_t relu_bwd(const float *y, const float *dy, float *dx, int64_t n, bool accumulate, hipStream_t s);
hipError_t add_fwd(const float *a, const float *b, float *z, int64_t n, hipStream_t s);
// z = max(a + b, 0)
hipError_t add_relu_fwd(const float *a, const float *b, float *z, int64_t n, hipStream_t s);
// m = dy where y > 0 else 0, written over dy; mode1 1: o1 = m, 2: o1 += m, 0: o1 unused
hipError_t add_relu_bwd(const float *y, float *dy, float *o1, int mode1, int64_t n, hipStream_t s);
// One bit per element of a ReLU output, "was it positive": bit e % 32 of word e / 32 (relu_mask_bytes(n) bytes, 16-byte aligned).
// The two backward kernels below take the mask in place of the output (same results: they only ever asked y > 0).
size_t relu_mask_bytes(int64_t n);
hipError_t relu_mask_pack(const float *y, uint32_t *mask, int64_t n, hipStream_t s);
hipError_t relu_bwd_mask(const uint32_t *mask, const float *dy, float *dx, int64_t n, bool accumulate, hipStream_t s);
hipError_t add_relu_bwd_mask(const uint32_t *mask, float *dy, float *o1, int mode1, int64_t n, hipStream_t s);
// dst += src
hipError_t accumulate(float *dst, const float *src, int64_t n, hipStream_t s);
hipError_t copy(float *dst, const float *src, int64_t n, hipStream_t s);

// plain SGD: p -= lr * g
hipError_t sgd_update(float *p, const float *g, float lr, int64_t n, hipStream_t s);
// crk[c][t][k] = krc[k][t][c]: refreshes the filter copy the data gradient reads
hipError_t filter_transpose(const float *krc, float *crk, int K, int64_t T, int C, hipStream_t s);

struct PoolGeom {
    int N, C, D, H, W, Do, Ho, Wo, kd, kh, kw, sd, sh, sw, pd, ph, pw;
};
hipError_t maxpool_fwd(const float *x, float *y, const PoolGeom &g, hipStream_t s);
hipError_t maxpool_bwd(const float *x, const float *dy, float *dx, const PoolGeom &g, bool accumulate, hipStream_t s);
// x[N][S][C] -> y[N][C]
hipError_t gavgpool_fwd(const float *x, float *y, int N, int64_t S, int C, hipStream_t s);
hipError_t gavgpool_bwd(const float *dy, float *dx, int N, int64_t S, int C, bool accumulate, hipStream_t s);

// y[n][o] += b[o];  db[o] = sum_n dy[n][o]
hipError_t bias_add(float *y, const float *b, int N, int O, hipStream_t s);
hipError_t bias_grad(const float *dy, float *db, int N, int O, hipStream_t s);

// loss[0] = mean_n (logsumexp(z_n) - z_n[t_n]); per_sample is N floats of scratch
hipError_t softmax_ce_fwd(const float *z, const int32_t *labels, float *per_sample, float *loss, int N, int K, hipStream_t s);
// dz (+)= (softmax(z) - onehot)/N
hipError_t softmax_ce_bwd(const float *z, const int32_t *labels, float *dz, int N, int K, bool accumulate, hipStream_t s);

}  // namespace pk
