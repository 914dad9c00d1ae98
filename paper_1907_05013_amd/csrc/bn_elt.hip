// HBM-bound layers for gfx950: batch normalisation (training mode) forward / backward and
// the element-wise layers (ReLU, residual add, gradient accumulate, copy).
//
// The paper (section 3.3) singles these out as layers of "small computation complexity":
// their time is memory traffic, so every kernel moves 16 bytes per lane per access over
// channels-last rows and touches each tensor the minimum number of times
// (BN forward: x twice + y once; BN backward: x, dy twice + dx once).
// Reductions are two-stage and fixed-order (per-thread strided partial sums -> in-block
// combine -> per-channel wavefront shuffle tree in double), so results are bit-identical
// from run to run and independent of where the tensor sits in the arena.
#include "kernels.h"

namespace pk {
namespace {

constexpr int BNT = 256;        // threads per block in the 2-d (row, channel-vector) kernels
constexpr int MAX_RBLK = 2048;  // cap on row blocks of a reduction
constexpr int APPLY_BLOCKS = 1 << 22;  // cap on blocks of an apply kernel

struct Lay2D {
    int V;          // floats per lane access (4 when C % 4 == 0, else 1)
    int CV;         // channel vectors per row
    int TX, TY;     // threads across channel vectors / rows
    int gy;         // blocks across channel vectors
    int nblk;       // row blocks
    int64_t rows_per_blk;
};

// rows_per_thread: how many rows one thread walks before its block is done.  The reductions take
// long walks (few partial results); the apply kernels take short ones: many small blocks, each
// streaming a few KB, measured closest to the HBM peak on this chip.
Lay2D layout2d(int64_t M, int C, bool vec_ok, int target_blocks, int rows_per_thread = 32)
{
    Lay2D L;
    L.V = (vec_ok && C % 4 == 0) ? 4 : 1;
    L.CV = C / L.V;
    L.TX = L.CV < BNT ? L.CV : BNT;
    L.TY = BNT / L.TX;
    L.gy = (L.CV + L.TX - 1) / L.TX;
    int64_t nb = (M + (int64_t)L.TY * rows_per_thread - 1) / ((int64_t)L.TY * rows_per_thread);
    int64_t cap = target_blocks / L.gy;
    if (cap < 1) cap = 1;
    if (nb > cap) nb = cap;
    if (nb < 1) nb = 1;
    L.rows_per_blk = (M + nb - 1) / nb;
    L.nblk = (int)((M + L.rows_per_blk - 1) / L.rows_per_blk);
    return L;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int V> __device__ __forceinline__ void ldv(const float *p, float (&o)[V])
{
    if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        o[0] = t.x; o[1 % V] = t.y; o[2 % V] = t.z; o[3 % V] = t.w;
    } else {
        o[0] = *p;
    }
}
template <int V> __device__ __forceinline__ void stv(float *p, const float (&o)[V])
{
    if constexpr (V == 4) *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1 % V], o[2 % V], o[3 % V]);
    else *p = o[0];
}
// Streaming accessors for the big tensors: every element is touched once per kernel, so the
// loads and stores carry the non-temporal hint and leave the caches to the per-channel vectors.
template <int V> __device__ __forceinline__ void ldnt(const float *p, float (&o)[V])
{
    if constexpr (V == 4) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        o[0] = t.x; o[1 % V] = t.y; o[2 % V] = t.z; o[3 % V] = t.w;
    } else {
        o[0] = __builtin_nontemporal_load(p);
    }
}
template <int V> __device__ __forceinline__ void stnt(float *p, const float (&o)[V])
{
    if constexpr (V == 4) {
        const f32x4 t = {o[0], o[1 % V], o[2 % V], o[3 % V]};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4 *>(p));
    } else {
        __builtin_nontemporal_store(o[0], p);
    }
}

// The one expression every kernel uses for a normalised value (g = gamma * istd): forward, the
// fused ReLU decision in forward and its re-derivation in backward all round identically.
__device__ __forceinline__ float bn_val(float x, float mu, float g, float b) { return __fmaf_rn(x - mu, g, b); }

// Stage 1 of both BN reductions.  part[blk][0][c] / part[blk][1][c]:
//   forward  (dy == nullptr): sum (x - x0_c), sum (x - x0_c)^2, x0_c = first row (a shift that
//                             keeps the variance formula from cancelling)
//   backward:                 sum dy, sum dy * (x - mean_c)
//   backward through a fused ReLU (RELU): dy is first masked by [bn_val(x) > 0]
template <int V, bool RELU>
__global__ __launch_bounds__(BNT) void bn_partial_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                          const float *__restrict__ mean, const float *__restrict__ gamma,
                                                          const float *__restrict__ beta, const float *__restrict__ istd,
                                                          float *__restrict__ part,
                                                          int64_t M, int C, int TX, int TY, int64_t rows_per_blk)
{
    __shared__ float red[2][BNT][V];
    const int tid = threadIdx.x;
    const int tx = tid % TX, ty = tid / TX;
    const int col = blockIdx.y * TX + tx;  // channel-vector index
    const bool active = ty < TY && col * V < C;
    float s1[V], s2[V];
#pragma unroll
    for (int i = 0; i < V; ++i) s1[i] = s2[i] = 0.f;
    if (active) {
        float sh[V], g[V], bt[V];
        ldv<V>((dy ? mean : x) + (int64_t)col * V, sh);
        if (RELU) {
            float is[V];
            ldv<V>(gamma + (int64_t)col * V, g);
            ldv<V>(istd + (int64_t)col * V, is);
            ldv<V>(beta + (int64_t)col * V, bt);
#pragma unroll
            for (int i = 0; i < V; ++i) g[i] *= is[i];
        }
        const int64_t r0 = (int64_t)blockIdx.x * rows_per_blk;
        const int64_t r1 = r0 + rows_per_blk < M ? r0 + rows_per_blk : M;
        auto take = [&](const float (&xv)[V], float (&dv)[V]) {
            if (dy) {
                if (RELU) {
#pragma unroll
                    for (int i = 0; i < V; ++i) dv[i] = bn_val(xv[i], sh[i], g[i], bt[i]) > 0.f ? dv[i] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < V; ++i) { s1[i] += dv[i]; s2[i] += dv[i] * (xv[i] - sh[i]); }
            } else {
#pragma unroll
                for (int i = 0; i < V; ++i) { const float d = xv[i] - sh[i]; s1[i] += d; s2[i] += d * d; }
            }
        };
        // UR rows in flight per thread; the sums still take the rows in ascending order
        constexpr int UR = 4;
        int64_t r = r0 + ty;
        for (; r + (int64_t)(UR - 1) * TY < r1; r += (int64_t)UR * TY) {
            float xv[UR][V], dv[UR][V];
#pragma unroll
            for (int u = 0; u < UR; ++u) ldnt<V>(x + (r + (int64_t)u * TY) * C + (int64_t)col * V, xv[u]);
            if (dy) {
#pragma unroll
                for (int u = 0; u < UR; ++u) ldnt<V>(dy + (r + (int64_t)u * TY) * C + (int64_t)col * V, dv[u]);
            }
#pragma unroll
            for (int u = 0; u < UR; ++u) take(xv[u], dv[u]);
        }
        for (; r < r1; r += TY) {
            float xv[V], dv[V];
            ldnt<V>(x + r * C + (int64_t)col * V, xv);
            if (dy) ldnt<V>(dy + r * C + (int64_t)col * V, dv);
            take(xv, dv);
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) { red[0][tid][i] = s1[i]; red[1][tid][i] = s2[i]; }
    __syncthreads();
    if (active && ty == 0) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            float a = red[0][tx][i], b = red[1][tx][i];
            for (int y = 1; y < TY; ++y) { a += red[0][y * TX + tx][i]; b += red[1][y * TX + tx][i]; }
            s1[i] = a; s2[i] = b;
        }
        stv<V>(part + ((int64_t)blockIdx.x * 2 + 0) * C + (int64_t)col * V, s1);
        stv<V>(part + ((int64_t)blockIdx.x * 2 + 1) * C + (int64_t)col * V, s2);
    }
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;  // lane 0 holds the total
}

// running averages: the batch mean, and the batch variance with the factor m / (m - 1) that makes it unbiased
__device__ __forceinline__ void run_update(const BnRun &run, int c, double mean, double var, double m)
{
    if (!run.mean) return;
    const double d = (double)run.decay, adjust = m / (m > 1.0 ? m - 1.0 : 1.0);
    run.mean[c] = (float)(d * (double)run.mean[c] + (1.0 - d) * mean);
    run.var[c] = (float)(d * (double)run.var[c] + (1.0 - d) * var * adjust);
}

// Stage 2: one wavefront per channel sums the row-block partials in double.
__global__ __launch_bounds__(64) void bn_stats_final_kernel(const float *__restrict__ part, const float *__restrict__ x,
                                                             float *__restrict__ mean, float *__restrict__ istd,
                                                             int nblk, int C, double m, double eps, BnRun run)
{
    const int c = blockIdx.x, lane = threadIdx.x;
    double a = 0.0, b = 0.0;
    for (int k = lane; k < nblk; k += 64) {
        a += (double)part[((int64_t)k * 2 + 0) * C + c];
        b += (double)part[((int64_t)k * 2 + 1) * C + c];
    }
    a = wave_sum(a);
    b = wave_sum(b);
    if (lane == 0) {
        const double d1 = a / m;
        double var = b / m - d1 * d1;
        if (var < 0.0) var = 0.0;
        mean[c] = (float)((double)x[c] + d1);
        istd[c] = (float)(1.0 / sqrt(var + eps));
        run_update(run, c, (double)x[c] + d1, var, m);
    }
}

// Statistics from per-tile (mean, M2) pairs: each lane merges every 64th tile in ascending order,
// then the 64 lane results are merged pairwise in a fixed tree -- all in double, by the update
// n = na + nb, d = mb - ma, mean = ma + d nb / n, M2 = M2a + M2b + d^2 na nb / n.
__global__ __launch_bounds__(64) void bn_tiles_final_kernel(const float *__restrict__ tiles, float *__restrict__ mean,
                                                             float *__restrict__ istd, int tiles_m, int rows_per_tile, int64_t M,
                                                             int C, double eps, BnRun run)
{
    const int c = blockIdx.x, lane = threadIdx.x;
    double n = 0.0, mu = 0.0, m2 = 0.0;
    for (int t = lane; t < tiles_m; t += 64) {
        int64_t rows = M - (int64_t)t * rows_per_tile;
        if (rows > rows_per_tile) rows = rows_per_tile;
        if (rows <= 0) continue;
        const double nb = (double)rows, mb = (double)tiles[((int64_t)t * 2 + 0) * C + c], qb = (double)tiles[((int64_t)t * 2 + 1) * C + c];
        const double tot = n + nb, d = mb - mu;
        mu += d * (nb / tot);
        m2 += qb + d * d * (n * nb / tot);
        n = tot;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double nb = __shfl_down(n, off, 64), mb = __shfl_down(mu, off, 64), qb = __shfl_down(m2, off, 64);
        if (nb > 0.0) {
            const double tot = n + nb, d = mb - mu;
            mu += d * (nb / tot);
            m2 += qb + d * d * (n * nb / tot);
            n = tot;
        }
    }
    if (lane == 0) {
        double var = m2 / (double)M;
        if (var < 0.0) var = 0.0;
        mean[c] = (float)mu;
        istd[c] = (float)(1.0 / sqrt(var + eps));
        run_update(run, c, mu, var, (double)M);
    }
}

// Coarsening of per-tile statistics: `group` consecutive tiles become one (the last group and the
// last tile may be short).  One block per (group, 64 channels); the four wavefronts take every
// fourth tile of the group.  Two passes over the few values involved, in double: the group's
// mean, then M2 = sum of (M2_t + n_t (mean_t - mean)^2); partial sums are combined in wavefront order.
__global__ __launch_bounds__(256) void bn_tiles_group_kernel(const float *__restrict__ tiles, float *__restrict__ out, int tiles_m,
                                                              int rows_per_tile, int group, int64_t M, int C)
{
    __shared__ double red[4][64];
    const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
    const int c = blockIdx.y * 64 + lane;
    const int t0 = blockIdx.x * group, t1 = min(tiles_m, t0 + group);
    const bool live = c < C;
    auto rows_of = [&](int t) {
        int64_t rows = M - (int64_t)t * rows_per_tile;
        return (double)(rows > rows_per_tile ? rows_per_tile : (rows < 0 ? 0 : rows));
    };
    double s = 0.0;
    if (live)
        for (int t = t0 + w; t < t1; t += 4) s += rows_of(t) * (double)tiles[((int64_t)t * 2 + 0) * C + c];
    red[w][lane] = s;
    __syncthreads();
    const double ng = rows_of(t0) + (t1 - t0 > 1 ? (double)(t1 - t0 - 2) * rows_per_tile + rows_of(t1 - 1) : 0.0);
    const double mu = ng > 0.0 ? (((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane]) / ng : 0.0;
    __syncthreads();
    double q = 0.0;
    for (int t = t0 + w; live && t < t1; t += 4) {
        const double nt = rows_of(t), d = (double)tiles[((int64_t)t * 2 + 0) * C + c] - mu;
        q += (double)tiles[((int64_t)t * 2 + 1) * C + c] + nt * d * d;
    }
    red[w][lane] = q;
    __syncthreads();
    if (w == 0 && live) {
        out[((int64_t)blockIdx.x * 2 + 0) * C + c] = (float)mu;
        out[((int64_t)blockIdx.x * 2 + 1) * C + c] = (float)(((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane]);
    }
}

// dbeta and dgamma from the per-row-block partial sums [nblk][2][C].  A block takes 16 channels: its 1024 threads are 64 groups
// of 16 lanes, group g adds the row blocks g, g + 64, ... of its lane's channel (16 consecutive channels per load: 64 contiguous
// bytes, where one wavefront per channel read 64 different cache lines per step), in double; the 64 group sums are then added in
// ascending order by the first group.
constexpr int GF_CH = 16, GF_GROUPS = 64;
__global__ __launch_bounds__(GF_CH * GF_GROUPS) void bn_grad_final_kernel(const float *__restrict__ part, const float *__restrict__ istd,
                                                                         float *__restrict__ dgamma, float *__restrict__ dbeta,
                                                                         int nblk, int C)
{
    __shared__ double ra[GF_GROUPS][GF_CH], rb[GF_GROUPS][GF_CH];
    const int tx = threadIdx.x % GF_CH, g = threadIdx.x / GF_CH;
    const int c = blockIdx.x * GF_CH + tx;
    double a = 0.0, b = 0.0;
    if (c < C) {
        // eight row blocks' values requested together, added in ascending order
        int k = g;
        for (; k + 7 * GF_GROUPS < nblk; k += 8 * GF_GROUPS) {
            float va[8], vb[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                va[u] = part[((int64_t)(k + u * GF_GROUPS) * 2 + 0) * C + c];
                vb[u] = part[((int64_t)(k + u * GF_GROUPS) * 2 + 1) * C + c];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                a += (double)va[u];
                b += (double)vb[u];
            }
        }
        for (; k < nblk; k += GF_GROUPS) {
            a += (double)part[((int64_t)k * 2 + 0) * C + c];
            b += (double)part[((int64_t)k * 2 + 1) * C + c];
        }
    }
    ra[g][tx] = a;
    rb[g][tx] = b;
    __syncthreads();
    if (g == 0 && c < C) {
        for (int j = 1; j < GF_GROUPS; ++j) {
            a += ra[j][tx];
            b += rb[j][tx];
        }
        dbeta[c] = (float)a;
        dgamma[c] = (float)(b * (double)istd[c]);
    }
}

// y = gamma * (x - mean) * istd + beta, optionally followed by ReLU
template <int V, bool RELU>
__global__ __launch_bounds__(BNT) void bn_apply_kernel(const float *__restrict__ x, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, const float *__restrict__ mean,
                                                        const float *__restrict__ istd, float *__restrict__ y,
                                                        int64_t M, int C, int TX, int TY, int64_t rows_per_blk)
{
    const int tid = threadIdx.x;
    const int tx = tid % TX, ty = tid / TX;
    const int col = blockIdx.y * TX + tx;
    if (ty >= TY || col * V >= C) return;
    float g[V], b[V], mu[V], is[V];
    ldv<V>(gamma + (int64_t)col * V, g);
    ldv<V>(beta + (int64_t)col * V, b);
    ldv<V>(mean + (int64_t)col * V, mu);
    ldv<V>(istd + (int64_t)col * V, is);
#pragma unroll
    for (int i = 0; i < V; ++i) g[i] *= is[i];
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_blk;
    const int64_t r1 = r0 + rows_per_blk < M ? r0 + rows_per_blk : M;
    auto apply = [&](float (&xv)[V]) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float v = bn_val(xv[i], mu[i], g[i], b[i]);
            xv[i] = RELU ? (v > 0.f ? v : 0.f) : v;
        }
    };
    constexpr int UR = 4;
    int64_t r = r0 + ty;
    for (; r + (int64_t)(UR - 1) * TY < r1; r += (int64_t)UR * TY) {
        float xv[UR][V];
#pragma unroll
        for (int u = 0; u < UR; ++u) ldnt<V>(x + (r + (int64_t)u * TY) * C + (int64_t)col * V, xv[u]);
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            apply(xv[u]);
            stnt<V>(y + (r + (int64_t)u * TY) * C + (int64_t)col * V, xv[u]);
        }
    }
    for (; r < r1; r += TY) {
        float xv[V];
        ldnt<V>(x + r * C + (int64_t)col * V, xv);
        apply(xv);
        stnt<V>(y + r * C + (int64_t)col * V, xv);
    }
}

// z = max(bn(x) + other, 0): the normalisation of a residual branch applied inside the add + ReLU that
// consumes it (bn(x) is rounded to fp32 before the add, exactly as when it is stored and re-read).
// BOTH: the other input is normalised here as well (a block whose shortcut is a projection):
// z = max(bn(x) + bn2(other), 0).
struct BnAffine {
    const float *gamma, *beta, *mean, *istd;
};

template <int V, bool BOTH>
__global__ __launch_bounds__(BNT) void bn_add_relu_kernel(const float *__restrict__ x, const float *__restrict__ other, BnAffine p,
                                                           BnAffine q, float *__restrict__ z, int64_t M, int C, int TX, int TY,
                                                           int64_t rows_per_blk)
{
    const int tid = threadIdx.x;
    const int tx = tid % TX, ty = tid / TX;
    const int col = blockIdx.y * TX + tx;
    if (ty >= TY || col * V >= C) return;
    float g[V], b[V], mu[V], is[V];
    ldv<V>(p.gamma + (int64_t)col * V, g);
    ldv<V>(p.beta + (int64_t)col * V, b);
    ldv<V>(p.mean + (int64_t)col * V, mu);
    ldv<V>(p.istd + (int64_t)col * V, is);
#pragma unroll
    for (int i = 0; i < V; ++i) g[i] *= is[i];
    float g2[V], b2[V], mu2[V];
    if (BOTH) {
        ldv<V>(q.gamma + (int64_t)col * V, g2);
        ldv<V>(q.beta + (int64_t)col * V, b2);
        ldv<V>(q.mean + (int64_t)col * V, mu2);
        ldv<V>(q.istd + (int64_t)col * V, is);
#pragma unroll
        for (int i = 0; i < V; ++i) g2[i] *= is[i];
    }
    auto combine = [&](float xv, float ov, int i) {
        const float o = BOTH ? bn_val(ov, mu2[i], g2[i], b2[i]) : ov;
        const float v = bn_val(xv, mu[i], g[i], b[i]) + o;
        return v > 0.f ? v : 0.f;
    };
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_blk;
    const int64_t r1 = r0 + rows_per_blk < M ? r0 + rows_per_blk : M;
    constexpr int UR = 2;
    int64_t r = r0 + ty;
    for (; r + (int64_t)(UR - 1) * TY < r1; r += (int64_t)UR * TY) {
        float xv[UR][V], ov[UR][V];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            ldnt<V>(x + (r + (int64_t)u * TY) * C + (int64_t)col * V, xv[u]);
            ldnt<V>(other + (r + (int64_t)u * TY) * C + (int64_t)col * V, ov[u]);
        }
#pragma unroll
        for (int u = 0; u < UR; ++u) {
#pragma unroll
            for (int i = 0; i < V; ++i) xv[u][i] = combine(xv[u][i], ov[u][i], i);
            stnt<V>(z + (r + (int64_t)u * TY) * C + (int64_t)col * V, xv[u]);
        }
    }
    for (; r < r1; r += TY) {
        float xv[V], ov[V];
        ldnt<V>(x + r * C + (int64_t)col * V, xv);
        ldnt<V>(other + r * C + (int64_t)col * V, ov);
#pragma unroll
        for (int i = 0; i < V; ++i) xv[i] = combine(xv[i], ov[i], i);
        stnt<V>(z + r * C + (int64_t)col * V, xv);
    }
}

// dx (+)= gamma*istd*(dy - dbeta/m - (x-mean)*istd*dgamma/m)
template <int V, bool ACCUM, bool RELU>
__global__ __launch_bounds__(BNT) void bn_bwd_apply_kernel(const float *__restrict__ x, const float *dy,
                                                            const float *__restrict__ gamma, const float *__restrict__ beta,
                                                            const float *__restrict__ mean,
                                                            const float *__restrict__ istd, const float *__restrict__ dgamma,
                                                            const float *__restrict__ dbeta, float *dx,
                                                            int64_t M, int C, int TX, int TY, int64_t rows_per_blk, float inv_m)
{
    const int tid = threadIdx.x;
    const int tx = tid % TX, ty = tid / TX;
    const int col = blockIdx.y * TX + tx;
    if (ty >= TY || col * V >= C) return;
    float a[V], b[V], cc[V], mu[V], bt[V];
    {
        float g[V], is[V], dg[V], db[V];
        ldv<V>(gamma + (int64_t)col * V, g);
        ldv<V>(istd + (int64_t)col * V, is);
        ldv<V>(dgamma + (int64_t)col * V, dg);
        ldv<V>(dbeta + (int64_t)col * V, db);
        ldv<V>(mean + (int64_t)col * V, mu);
        if (RELU) ldv<V>(beta + (int64_t)col * V, bt);
#pragma unroll
        for (int i = 0; i < V; ++i) { a[i] = g[i] * is[i]; b[i] = db[i] * inv_m; cc[i] = is[i] * dg[i] * inv_m; }
    }
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_blk;
    const int64_t r1 = r0 + rows_per_blk < M ? r0 + rows_per_blk : M;
    auto grad = [&](const float (&xv)[V], float (&dv)[V]) {
        if (RELU) {
#pragma unroll
            for (int i = 0; i < V; ++i) dv[i] = bn_val(xv[i], mu[i], a[i], bt[i]) > 0.f ? dv[i] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < V; ++i) dv[i] = a[i] * (dv[i] - b[i] - (xv[i] - mu[i]) * cc[i]);
    };
    constexpr int UR = 2;
    int64_t r = r0 + ty;
    for (; r + (int64_t)(UR - 1) * TY < r1; r += (int64_t)UR * TY) {
        float xv[UR][V], dv[UR][V], ov[UR][V];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            ldnt<V>(x + (r + (int64_t)u * TY) * C + (int64_t)col * V, xv[u]);
            ldnt<V>(dy + (r + (int64_t)u * TY) * C + (int64_t)col * V, dv[u]);
            if (ACCUM) ldnt<V>(dx + (r + (int64_t)u * TY) * C + (int64_t)col * V, ov[u]);
        }
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            grad(xv[u], dv[u]);
            if (ACCUM) {
#pragma unroll
                for (int i = 0; i < V; ++i) dv[u][i] = ov[u][i] + dv[u][i];
            }
            stnt<V>(dx + (r + (int64_t)u * TY) * C + (int64_t)col * V, dv[u]);
        }
    }
    for (; r < r1; r += TY) {
        float xv[V], dv[V];
        ldnt<V>(x + r * C + (int64_t)col * V, xv);
        ldnt<V>(dy + r * C + (int64_t)col * V, dv);
        grad(xv, dv);
        if (ACCUM) {
            float ov[V];
            ldnt<V>(dx + r * C + (int64_t)col * V, ov);
#pragma unroll
            for (int i = 0; i < V; ++i) dv[i] = ov[i] + dv[i];
        }
        stnt<V>(dx + r * C + (int64_t)col * V, dv);
    }
}

// ---- flat element-wise kernels: n4 float4 items then a scalar tail ----
enum { EW_RELU_F, EW_RELU_B, EW_RELU_B_ACC, EW_ADD, EW_ACC, EW_COPY, EW_ADD_RELU };

template <int OP> __device__ __forceinline__ float ew(float a, float b, float d)
{
    switch (OP) {
    case EW_RELU_F: return a > 0.f ? a : 0.f;            // a = x
    case EW_RELU_B: return a > 0.f ? b : 0.f;            // a = y, b = dy
    case EW_RELU_B_ACC: return d + (a > 0.f ? b : 0.f);  // d = existing dx
    case EW_ADD: return a + b;
    case EW_ADD_RELU: { const float z = a + b; return z > 0.f ? z : 0.f; }
    case EW_ACC: return d + a;                           // a = src
    default: return a;
    }
}

// One float4 per thread and no loop: many short-lived blocks, each streaming 4 KB per tensor.
template <int OP>
__global__ __launch_bounds__(256) void ew_kernel(const float *a, const float *b, float *d, int64_t n)
{
    constexpr bool USE_B = OP == EW_RELU_B || OP == EW_RELU_B_ACC || OP == EW_ADD || OP == EW_ADD_RELU;
    constexpr bool USE_D = OP == EW_RELU_B_ACC || OP == EW_ACC;
    const int64_t n4 = n / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const f32x4 av = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a) + i);
        f32x4 bv = {0.f, 0.f, 0.f, 0.f}, dv = bv;
        if (USE_B) bv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(b) + i);
        if (USE_D) dv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(d) + i);
        f32x4 o;
        o.x = ew<OP>(av.x, bv.x, dv.x);
        o.y = ew<OP>(av.y, bv.y, dv.y);
        o.z = ew<OP>(av.z, bv.z, dv.z);
        o.w = ew<OP>(av.w, bv.w, dv.w);
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(d) + i);
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
        const int64_t t = n4 * 4 + threadIdx.x;
        d[t] = ew<OP>(a[t], USE_B ? b[t] : 0.f, USE_D ? d[t] : 0.f);
    }
}

// blocks of a one-float4-per-thread launch over n floats
unsigned ew_blocks(int64_t n)
{
    const int64_t blocks = (n / 4 + 255) / 256;
    return (unsigned)(blocks < 1 ? 1 : blocks);
}

template <int OP> hipError_t launch_ew(const float *a, const float *b, float *d, int64_t n, hipStream_t s)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || !a || !d) return hipErrorInvalidValue;
    if (n == 0) return hipSuccess;
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)d) % 16 != 0) return hipErrorInvalidValue;
    ew_kernel<OP><<<dim3(ew_blocks(n)), dim3(256), 0, s>>>(a, b, d, n);
    return hipGetLastError();
}

// backward of y = relu(a + b): m = dy where y > 0 else 0; m overwrites dy (the gradient of one
// input takes over that buffer) and, when o1 is given, is written (mode 1) or added (mode 2) there
template <int MODE1>
__global__ __launch_bounds__(256) void addrelu_bwd_kernel(const float *__restrict__ y, float *dy, float *o1, int64_t n)
{
    const int64_t n4 = n / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const f32x4 yv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(y) + i);
        f32x4 d = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(dy) + i);
        f32x4 e = {0.f, 0.f, 0.f, 0.f};
        if (MODE1 == 2) e = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(o1) + i);
        d.x = yv.x > 0.f ? d.x : 0.f; d.y = yv.y > 0.f ? d.y : 0.f; d.z = yv.z > 0.f ? d.z : 0.f; d.w = yv.w > 0.f ? d.w : 0.f;
        __builtin_nontemporal_store(d, reinterpret_cast<f32x4 *>(dy) + i);
        if (MODE1 == 1) __builtin_nontemporal_store(d, reinterpret_cast<f32x4 *>(o1) + i);
        if (MODE1 == 2) {
            e.x += d.x; e.y += d.y; e.z += d.z; e.w += d.w;
            __builtin_nontemporal_store(e, reinterpret_cast<f32x4 *>(o1) + i);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
        const int64_t t = n4 * 4 + threadIdx.x;
        const float d = y[t] > 0.f ? dy[t] : 0.f;
        dy[t] = d;
        if (MODE1 == 1) o1[t] = d;
        if (MODE1 == 2) o1[t] += d;
    }
}

// ---- one-bit ReLU masks ----
// Thread i owns elements 4 i .. 4 i + 3 (the thread after the last whole group owns the tail of up to three); its four bits
// go to position 4 (i % 8) of word i / 8, so bit e % 32 of word e / 32 says whether element e was positive.
__global__ __launch_bounds__(256) void relu_mask_pack_kernel(const float *__restrict__ y, uint32_t *__restrict__ mask, int64_t n)
{
    const int64_t n4 = n / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t nib = 0;
    if (i < n4) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(y) + i);
        nib = (v.x > 0.f ? 1u : 0u) | (v.y > 0.f ? 2u : 0u) | (v.z > 0.f ? 4u : 0u) | (v.w > 0.f ? 8u : 0u);
    } else if (i == n4) {
        for (int t = 0; t < (int)(n - n4 * 4); ++t) nib |= (y[n4 * 4 + t] > 0.f ? 1u : 0u) << t;
    }
    // the eight threads of a word are eight consecutive lanes of one wavefront (256 threads per block, i % 8 == lane % 8)
    uint32_t w = nib << (4 * (threadIdx.x & 7));
    w |= __shfl_xor(w, 1, 64);
    w |= __shfl_xor(w, 2, 64);
    w |= __shfl_xor(w, 4, 64);
    if ((threadIdx.x & 7) == 0 && i * 4 < n) mask[i / 8] = w;
}

__device__ __forceinline__ uint32_t mask_nibble(const uint32_t *__restrict__ mask, int64_t i)
{
    return (mask[i / 8] >> (4 * (int)(i & 7))) & 15u;
}
__device__ __forceinline__ bool mask_bit(const uint32_t *__restrict__ mask, int64_t e) { return (mask[e / 32] >> (int)(e & 31)) & 1u; }

// dx (+)= dy where the mask is set
template <bool ACC>
__global__ __launch_bounds__(256) void relu_bwd_mask_kernel(const uint32_t *__restrict__ mask, const float *dy, float *dx, int64_t n)
{
    const int64_t n4 = n / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const uint32_t nib = mask_nibble(mask, i);
        f32x4 d = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(dy) + i);
        d.x = (nib & 1u) ? d.x : 0.f; d.y = (nib & 2u) ? d.y : 0.f; d.z = (nib & 4u) ? d.z : 0.f; d.w = (nib & 8u) ? d.w : 0.f;
        if (ACC) d += __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(dx) + i);
        __builtin_nontemporal_store(d, reinterpret_cast<f32x4 *>(dx) + i);
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
        const int64_t t = n4 * 4 + threadIdx.x;
        const float d = mask_bit(mask, t) ? dy[t] : 0.f;
        dx[t] = ACC ? dx[t] + d : d;
    }
}

// addrelu_bwd_kernel with the mask in place of y
template <int MODE1>
__global__ __launch_bounds__(256) void addrelu_bwd_mask_kernel(const uint32_t *__restrict__ mask, float *dy, float *o1, int64_t n)
{
    const int64_t n4 = n / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const uint32_t nib = mask_nibble(mask, i);
        f32x4 d = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(dy) + i);
        f32x4 e = {0.f, 0.f, 0.f, 0.f};
        if (MODE1 == 2) e = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(o1) + i);
        d.x = (nib & 1u) ? d.x : 0.f; d.y = (nib & 2u) ? d.y : 0.f; d.z = (nib & 4u) ? d.z : 0.f; d.w = (nib & 8u) ? d.w : 0.f;
        __builtin_nontemporal_store(d, reinterpret_cast<f32x4 *>(dy) + i);
        if (MODE1 == 1) __builtin_nontemporal_store(d, reinterpret_cast<f32x4 *>(o1) + i);
        if (MODE1 == 2) {
            e.x += d.x; e.y += d.y; e.z += d.z; e.w += d.w;
            __builtin_nontemporal_store(e, reinterpret_cast<f32x4 *>(o1) + i);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
        const int64_t t = n4 * 4 + threadIdx.x;
        const float d = mask_bit(mask, t) ? dy[t] : 0.f;
        dy[t] = d;
        if (MODE1 == 1) o1[t] = d;
        if (MODE1 == 2) o1[t] += d;
    }
}

// p -= lr * g
__global__ __launch_bounds__(256) void sgd_kernel(float *__restrict__ p, const float *__restrict__ g, float lr, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = p[i] - lr * g[i];
}

// filter copy for the data gradient: crk[c][t][k] = krc[k][t][c]
__global__ __launch_bounds__(256) void filter_transpose_kernel(const float *__restrict__ krc, float *__restrict__ crk, int K, int64_t T, int C)
{
    const int64_t n = (int64_t)K * T * C;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int k = (int)(i % K);
        const int64_t ct = i / K;
        const int64_t t = ct % T;
        const int c = (int)(ct / T);
        crk[i] = krc[((int64_t)k * T + t) * C + c];
    }
}

bool bn_args_ok(int64_t M, int C) { return M > 0 && C > 0 && M * (int64_t)C < ((int64_t)1 << 40); }

}  // namespace

namespace {
// tiles folded into one before the final per-channel merge (1: none)
int bn_tiles_group(int tiles_m) { return tiles_m > 1024 ? (tiles_m + 511) / 512 : 1; }
}  // namespace

size_t bn_tiles_workspace_floats(int tiles_m, int C)
{
    if (tiles_m <= 0 || C <= 0) return 0;
    const int group = bn_tiles_group(tiles_m);
    const size_t groups = group > 1 ? (size_t)(tiles_m + group - 1) / group : 0;
    return (size_t)2 * C * ((size_t)tiles_m + groups);
}

size_t bn_workspace_floats(int64_t M, int C)
{
    if (!bn_args_ok(M, C)) return 0;
    const Lay2D a = layout2d(M, C, true, MAX_RBLK), b = layout2d(M, C, false, MAX_RBLK);
    return (size_t)(a.nblk > b.nblk ? a.nblk : b.nblk) * 2 * C;
}

hipError_t bn_apply(const float *x, const float *gamma, const float *beta, const float *mean, const float *istd,
                    float *y, int64_t M, int C, bool relu, hipStream_t s)
{
    if (!x || !gamma || !beta || !mean || !istd || !y || !bn_args_ok(M, C)) return hipErrorInvalidValue;
    const bool al = ((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma | (uintptr_t)beta | (uintptr_t)mean | (uintptr_t)istd) % 16 == 0;
    const Lay2D L = layout2d(M, C, al, APPLY_BLOCKS, 4);
    const dim3 grid(L.nblk, L.gy), block(BNT);
#define APPLY(V, R) bn_apply_kernel<V, R><<<grid, block, 0, s>>>(x, gamma, beta, mean, istd, y, M, C, L.TX, L.TY, L.rows_per_blk)
    if (L.V == 4) { if (relu) APPLY(4, true); else APPLY(4, false); }
    else { if (relu) APPLY(1, true); else APPLY(1, false); }
#undef APPLY
    return hipGetLastError();
}

hipError_t bn_stats(const float *x, float *mean, float *istd, float *ws, int64_t M, int C, float eps, BnRun run, hipStream_t s)
{
    if (!x || !mean || !istd || !ws || !bn_args_ok(M, C) || !run.mean != !run.var) return hipErrorInvalidValue;
    const bool al = ((uintptr_t)x | (uintptr_t)ws | (uintptr_t)mean) % 16 == 0;
    Lay2D L = layout2d(M, C, al, MAX_RBLK);
    const dim3 grid(L.nblk, L.gy), block(BNT);
    if (L.V == 4) bn_partial_kernel<4, false><<<grid, block, 0, s>>>(x, nullptr, nullptr, nullptr, nullptr, nullptr, ws, M, C, L.TX, L.TY, L.rows_per_blk);
    else bn_partial_kernel<1, false><<<grid, block, 0, s>>>(x, nullptr, nullptr, nullptr, nullptr, nullptr, ws, M, C, L.TX, L.TY, L.rows_per_blk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bn_stats_final_kernel<<<dim3(C), dim3(64), 0, s>>>(ws, x, mean, istd, L.nblk, C, (double)M, (double)eps, run);
    return hipGetLastError();
}

hipError_t bn_fwd(const float *x, const float *gamma, const float *beta, float *y, float *mean, float *istd,
                  float *ws, int64_t M, int C, float eps, bool relu, BnRun run, hipStream_t s)
{
    if (!gamma || !beta || !y) return hipErrorInvalidValue;
    const hipError_t e = bn_stats(x, mean, istd, ws, M, C, eps, run, s);
    if (e != hipSuccess) return e;
    return bn_apply(x, gamma, beta, mean, istd, y, M, C, relu, s);
}

hipError_t bn_add_relu_fwd(const float *x, const float *other, const float *gamma, const float *beta, const float *mean,
                           const float *istd, const float *gamma2, const float *beta2, const float *mean2, const float *istd2,
                           float *z, int64_t M, int C, hipStream_t s)
{
    if (!x || !other || !gamma || !beta || !mean || !istd || !z || !bn_args_ok(M, C)) return hipErrorInvalidValue;
    const bool both = gamma2 != nullptr;
    if (both ? (!beta2 || !mean2 || !istd2) : (beta2 || mean2 || istd2)) return hipErrorInvalidValue;
    const bool al = ((uintptr_t)x | (uintptr_t)other | (uintptr_t)z | (uintptr_t)gamma | (uintptr_t)beta | (uintptr_t)mean |
                     (uintptr_t)istd | (uintptr_t)gamma2 | (uintptr_t)beta2 | (uintptr_t)mean2 | (uintptr_t)istd2) % 16 == 0;
    const Lay2D L = layout2d(M, C, al, APPLY_BLOCKS, 4);
    const dim3 grid(L.nblk, L.gy), block(BNT);
    const BnAffine p{gamma, beta, mean, istd}, q{gamma2, beta2, mean2, istd2};
#define BN_ADD_RELU(V, BOTH) bn_add_relu_kernel<V, BOTH><<<grid, block, 0, s>>>(x, other, p, q, z, M, C, L.TX, L.TY, L.rows_per_blk)
    if (L.V == 4) { if (both) BN_ADD_RELU(4, true); else BN_ADD_RELU(4, false); }
    else { if (both) BN_ADD_RELU(1, true); else BN_ADD_RELU(1, false); }
#undef BN_ADD_RELU
    return hipGetLastError();
}

hipError_t bn_stats_from_tiles(float *tiles, int tiles_m, int rows_per_tile, int64_t M, int C, float eps, float *mean, float *istd,
                               BnRun run, hipStream_t s)
{
    if (!mean || !istd || !tiles || !bn_args_ok(M, C) || !run.mean != !run.var) return hipErrorInvalidValue;
    if (tiles_m <= 0 || rows_per_tile <= 0 || (int64_t)tiles_m * rows_per_tile < M || (int64_t)(tiles_m - 1) * rows_per_tile >= M)
        return hipErrorInvalidValue;
    const int group = bn_tiles_group(tiles_m);
    if (group > 1) {
        // many tiles: first fold groups of them, so that the per-channel wavefronts below have little to walk
        const int groups = (tiles_m + group - 1) / group;
        float *folded = tiles + (size_t)2 * tiles_m * C;
        bn_tiles_group_kernel<<<dim3(groups, (C + 63) / 64), dim3(256), 0, s>>>(tiles, folded, tiles_m, rows_per_tile, group, M, C);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        bn_tiles_final_kernel<<<dim3(C), dim3(64), 0, s>>>(folded, mean, istd, groups, rows_per_tile * group, M, C, (double)eps, run);
    } else {
        bn_tiles_final_kernel<<<dim3(C), dim3(64), 0, s>>>(tiles, mean, istd, tiles_m, rows_per_tile, M, C, (double)eps, run);
    }
    return hipGetLastError();
}

hipError_t bn_fwd_from_tiles(const float *x, const float *gamma, const float *beta, float *y, float *mean, float *istd,
                             float *tiles, int tiles_m, int rows_per_tile, int64_t M, int C, float eps, bool relu, BnRun run,
                             hipStream_t s)
{
    if (!x || !gamma || !beta || !y) return hipErrorInvalidValue;
    const hipError_t e = bn_stats_from_tiles(tiles, tiles_m, rows_per_tile, M, C, eps, mean, istd, run, s);
    if (e != hipSuccess) return e;
    return bn_apply(x, gamma, beta, mean, istd, y, M, C, relu, s);
}

hipError_t bn_bwd(const float *x, const float *dy, const float *gamma, const float *beta, const float *mean, const float *istd,
                  float *dx, float *dgamma, float *dbeta, float *ws, int64_t M, int C, bool accumulate, bool relu, hipStream_t s)
{
    if (!x || !dy || !gamma || !beta || !mean || !istd || !dgamma || !dbeta || !ws || !bn_args_ok(M, C)) return hipErrorInvalidValue;
    const bool al = ((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx | (uintptr_t)ws | (uintptr_t)mean | (uintptr_t)istd |
                     (uintptr_t)gamma | (uintptr_t)dgamma | (uintptr_t)dbeta) % 16 == 0;
    Lay2D L = layout2d(M, C, al, MAX_RBLK);
    {
        const dim3 grid(L.nblk, L.gy), block(BNT);
#define PARTIAL(V, R) bn_partial_kernel<V, R><<<grid, block, 0, s>>>(x, dy, mean, gamma, beta, istd, ws, M, C, L.TX, L.TY, L.rows_per_blk)
        if (L.V == 4) { if (relu) PARTIAL(4, true); else PARTIAL(4, false); }
        else { if (relu) PARTIAL(1, true); else PARTIAL(1, false); }
#undef PARTIAL
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        bn_grad_final_kernel<<<dim3((C + GF_CH - 1) / GF_CH), dim3(GF_CH * GF_GROUPS), 0, s>>>(ws, istd, dgamma, dbeta, L.nblk, C);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!dx) return hipSuccess;   // the input's gradient is not wanted: dgamma and dbeta only, dy stays as it is
    L = layout2d(M, C, al, APPLY_BLOCKS, 4);
    const dim3 grid(L.nblk, L.gy), block(BNT);
    const float inv_m = (float)(1.0 / (double)M);
#define BWD_APPLY(V, A, R) bn_bwd_apply_kernel<V, A, R><<<grid, block, 0, s>>>(x, dy, gamma, beta, mean, istd, dgamma, dbeta, dx, M, C, L.TX, L.TY, L.rows_per_blk, inv_m)
#define BWD_APPLY2(V, A) do { if (relu) BWD_APPLY(V, A, true); else BWD_APPLY(V, A, false); } while (0)
    if (L.V == 4) { if (accumulate) BWD_APPLY2(4, true); else BWD_APPLY2(4, false); }
    else { if (accumulate) BWD_APPLY2(1, true); else BWD_APPLY2(1, false); }
#undef BWD_APPLY2
#undef BWD_APPLY
    return hipGetLastError();
}

hipError_t relu_fwd(const float *x, float *y, int64_t n, hipStream_t s) { return launch_ew<EW_RELU_F>(x, nullptr, y, n, s); }
hipError_t relu_bwd(const float *y, const float *dy, float *dx, int64_t n, bool accumulate, hipStream_t s)
{
    if (!dy) return hipErrorInvalidValue;
    return accumulate ? launch_ew<EW_RELU_B_ACC>(y, dy, dx, n, s) : launch_ew<EW_RELU_B>(y, dy, dx, n, s);
}
hipError_t add_fwd(const float *a, const float *b, float *z, int64_t n, hipStream_t s)
{
    if (!b) return hipErrorInvalidValue;
    return launch_ew<EW_ADD>(a, b, z, n, s);
}
hipError_t add_relu_fwd(const float *a, const float *b, float *z, int64_t n, hipStream_t s)
{
    if (!b) return hipErrorInvalidValue;
    return launch_ew<EW_ADD_RELU>(a, b, z, n, s);
}
hipError_t add_relu_bwd(const float *y, float *dy, float *o1, int mode1, int64_t n, hipStream_t s)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || !y || !dy || (mode1 != 0 && !o1) || mode1 < 0 || mode1 > 2) return hipErrorInvalidValue;
    if (n == 0) return hipSuccess;
    if (((uintptr_t)y | (uintptr_t)dy | (uintptr_t)o1) % 16 != 0) return hipErrorInvalidValue;
    const dim3 grid(ew_blocks(n)), block(256);
    if (mode1 == 0) addrelu_bwd_kernel<0><<<grid, block, 0, s>>>(y, dy, o1, n);
    else if (mode1 == 1) addrelu_bwd_kernel<1><<<grid, block, 0, s>>>(y, dy, o1, n);
    else addrelu_bwd_kernel<2><<<grid, block, 0, s>>>(y, dy, o1, n);
    return hipGetLastError();
}
size_t relu_mask_bytes(int64_t n) { return n <= 0 ? 0 : (size_t)((n + 31) / 32) * 4; }
hipError_t relu_mask_pack(const float *y, uint32_t *mask, int64_t n, hipStream_t s)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || !y || !mask) return hipErrorInvalidValue;
    if (n == 0) return hipSuccess;
    if (((uintptr_t)y | (uintptr_t)mask) % 16 != 0) return hipErrorInvalidValue;
    const int64_t threads = (n + 3) / 4;   // one per group of four, the last of them for the tail
    relu_mask_pack_kernel<<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s>>>(y, mask, n);
    return hipGetLastError();
}
hipError_t relu_bwd_mask(const uint32_t *mask, const float *dy, float *dx, int64_t n, bool accumulate, hipStream_t s)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || !mask || !dy || !dx) return hipErrorInvalidValue;
    if (n == 0) return hipSuccess;
    if (((uintptr_t)mask | (uintptr_t)dy | (uintptr_t)dx) % 16 != 0) return hipErrorInvalidValue;
    const dim3 grid(ew_blocks(n)), block(256);
    if (accumulate) relu_bwd_mask_kernel<true><<<grid, block, 0, s>>>(mask, dy, dx, n);
    else relu_bwd_mask_kernel<false><<<grid, block, 0, s>>>(mask, dy, dx, n);
    return hipGetLastError();
}
hipError_t add_relu_bwd_mask(const uint32_t *mask, float *dy, float *o1, int mode1, int64_t n, hipStream_t s)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || !mask || !dy || (mode1 != 0 && !o1) || mode1 < 0 || mode1 > 2) return hipErrorInvalidValue;
    if (n == 0) return hipSuccess;
    if (((uintptr_t)mask | (uintptr_t)dy | (uintptr_t)o1) % 16 != 0) return hipErrorInvalidValue;
    const dim3 grid(ew_blocks(n)), block(256);
    if (mode1 == 0) addrelu_bwd_mask_kernel<0><<<grid, block, 0, s>>>(mask, dy, o1, n);
    else if (mode1 == 1) addrelu_bwd_mask_kernel<1><<<grid, block, 0, s>>>(mask, dy, o1, n);
    else addrelu_bwd_mask_kernel<2><<<grid, block, 0, s>>>(mask, dy, o1, n);
    return hipGetLastError();
}
hipError_t sgd_update(float *p, const float *g, float lr, int64_t n, hipStream_t s)
{
    if (!p || !g || n <= 0) return hipErrorInvalidValue;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    sgd_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(p, g, lr, n);
    return hipGetLastError();
}
hipError_t filter_transpose(const float *krc, float *crk, int K, int64_t T, int C, hipStream_t s)
{
    if (!krc || !crk || K <= 0 || T <= 0 || C <= 0) return hipErrorInvalidValue;
    int64_t blocks = ((int64_t)K * T * C + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    filter_transpose_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(krc, crk, K, T, C);
    return hipGetLastError();
}
hipError_t accumulate(float *dst, const float *src, int64_t n, hipStream_t s) { return launch_ew<EW_ACC>(src, nullptr, dst, n, s); }
hipError_t copy(float *dst, const float *src, int64_t n, hipStream_t s) { return launch_ew<EW_COPY>(src, nullptr, dst, n, s); }

}  // namespace pk
