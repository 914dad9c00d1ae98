// Pooling, global average pooling, FC bias and softmax cross-entropy kernels for gfx950.
// Channels-last tensors: consecutive lanes take consecutive channels, so every access of a
// wavefront is one contiguous run.  No atomics anywhere: the max-pool gradient is a gather
// (each input element visits the windows that contain it in scan order), which makes it
// deterministic and gives the same summation order as scattering window by window.
#include "kernels.h"

#include <cstdlib>

namespace pk {
namespace {

// first maximal in-bounds element (scan order d,h,w) of window (od,oh,ow) for channel c of image n
__device__ __forceinline__ void window_argmax(const float *__restrict__ x, const PoolGeom &g, int n, int od, int oh, int ow, int c,
                                              float &best, int &bd, int &bh, int &bw)
{
    bd = -1; bh = -1; bw = -1;
    best = -INFINITY;
    for (int a = 0; a < g.kd; ++a) {
        const int id = od * g.sd - g.pd + a;
        if ((unsigned)id >= (unsigned)g.D) continue;
        for (int b = 0; b < g.kh; ++b) {
            const int ih = oh * g.sh - g.ph + b;
            if ((unsigned)ih >= (unsigned)g.H) continue;
            for (int e = 0; e < g.kw; ++e) {
                const int iw = ow * g.sw - g.pw + e;
                if ((unsigned)iw >= (unsigned)g.W) continue;
                const float v = x[((((int64_t)n * g.D + id) * g.H + ih) * g.W + iw) * g.C + c];
                if (bd < 0 || v > best) { best = v; bd = id; bh = ih; bw = iw; }
            }
        }
    }
}

__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, PoolGeom g, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % g.C);
    int64_t t = i / g.C;
    const int ow = (int)(t % g.Wo); t /= g.Wo;
    const int oh = (int)(t % g.Ho); t /= g.Ho;
    const int od = (int)(t % g.Do);
    const int n = (int)(t / g.Do);
    float best; int bd, bh, bw;
    window_argmax(x, g, n, od, oh, ow, c, best, bd, bh, bw);
    y[i] = best;
}

// Workgroups are dealt to the eight XCDs in turn, and each XCD has an L2 of its own.  Overlapping pool windows make
// neighbouring workgroups read the same input rows; with `spread` (a grid of 8 * spread workgroups) each XCD takes a
// contiguous eighth of the index space, so those rows are fetched from memory once instead of once per XCD that meets them.
__device__ __forceinline__ int64_t pool_block(unsigned spread)
{
    return spread ? (int64_t)(blockIdx.x % 8) * spread + blockIdx.x / 8 : (int64_t)blockIdx.x;
}

// Four channels per thread (C % 4 == 0): the same scan order and the same strict comparison per
// channel as the scalar kernel, with 16-byte accesses.
__global__ __launch_bounds__(256) void maxpool_fwd_vec4_kernel(const float *__restrict__ x, float *__restrict__ y, PoolGeom g, int64_t total4,
                                                               unsigned spread)
{
    const int64_t i = pool_block(spread) * blockDim.x + threadIdx.x;
    if (i >= total4) return;
    const int C4 = g.C / 4;
    const int c = (int)(i % C4) * 4;
    int64_t t = i / C4;
    const int ow = (int)(t % g.Wo); t /= g.Wo;
    const int oh = (int)(t % g.Ho); t /= g.Ho;
    const int od = (int)(t % g.Do);
    const int n = (int)(t / g.Do);
    float4 best = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    bool first = true;
    for (int a = 0; a < g.kd; ++a) {
        const int id = od * g.sd - g.pd + a;
        if ((unsigned)id >= (unsigned)g.D) continue;
        for (int b = 0; b < g.kh; ++b) {
            const int ih = oh * g.sh - g.ph + b;
            if ((unsigned)ih >= (unsigned)g.H) continue;
            for (int e = 0; e < g.kw; ++e) {
                const int iw = ow * g.sw - g.pw + e;
                if ((unsigned)iw >= (unsigned)g.W) continue;
                const float4 v = *reinterpret_cast<const float4 *>(x + ((((int64_t)n * g.D + id) * g.H + ih) * g.W + iw) * g.C + c);
                if (first) { best = v; first = false; }
                else {
                    if (v.x > best.x) best.x = v.x;
                    if (v.y > best.y) best.y = v.y;
                    if (v.z > best.z) best.z = v.z;
                    if (v.w > best.w) best.w = v.w;
                }
            }
        }
    }
    *reinterpret_cast<float4 *>(y + i * 4) = best;
}

__device__ __forceinline__ int ceil_div_pos(int a, int b) { return a <= 0 ? 0 : (a + b - 1) / b; }

template <bool ACCUM>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dy, float *dx, PoolGeom g, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % g.C);
    int64_t t = i / g.C;
    const int iw = (int)(t % g.W); t /= g.W;
    const int ih = (int)(t % g.H); t /= g.H;
    const int id = (int)(t % g.D);
    const int n = (int)(t / g.D);
    // windows o with o*s - p <= i <= o*s - p + k - 1
    const int od0 = ceil_div_pos(id + g.pd - g.kd + 1, g.sd), od1 = min(g.Do - 1, (id + g.pd) / g.sd);
    const int oh0 = ceil_div_pos(ih + g.ph - g.kh + 1, g.sh), oh1 = min(g.Ho - 1, (ih + g.ph) / g.sh);
    const int ow0 = ceil_div_pos(iw + g.pw - g.kw + 1, g.sw), ow1 = min(g.Wo - 1, (iw + g.pw) / g.sw);
    float acc = 0.f;
    for (int od = od0; od <= od1; ++od)
        for (int oh = oh0; oh <= oh1; ++oh)
            for (int ow = ow0; ow <= ow1; ++ow) {
                float best; int bd, bh, bw;
                window_argmax(x, g, n, od, oh, ow, c, best, bd, bh, bw);
                if (bd == id && bh == ih && bw == iw)
                    acc += dy[((((int64_t)n * g.Do + od) * g.Ho + oh) * g.Wo + ow) * g.C + c];
            }
    dx[i] = ACCUM ? dx[i] + acc : acc;
}

// 2-d 3x3 window, stride 2, padding 1 (the ResNet stem pool), C % 4 == 0.  One thread owns the
// 2x2 block of input positions (2a..2a+1, 2b..2b+1) of four channels.  Only the windows
// (a..a+1, b..b+1) reach that block; their union is a 5x5 patch, loaded once.
template <bool ACCUM>
__global__ __launch_bounds__(256) void maxpool_k3s2p1_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dy, float *dx,
                                                                  PoolGeom g, int HB, int WB, int64_t total, unsigned spread)
{
    const int64_t i = pool_block(spread) * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int C4 = g.C / 4;
    const int c = (int)(i % C4) * 4;
    int64_t t = i / C4;
    const int b = (int)(t % WB); t /= WB;
    const int a = (int)(t % HB);
    const int n = (int)(t / HB);
    float4 patch[5][5];
    bool rv[5], cv[5];
#pragma unroll
    for (int r = 0; r < 5; ++r) { rv[r] = (unsigned)(2 * a - 1 + r) < (unsigned)g.H; cv[r] = (unsigned)(2 * b - 1 + r) < (unsigned)g.W; }
#pragma unroll
    for (int r = 0; r < 5; ++r)
#pragma unroll
        for (int q = 0; q < 5; ++q) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rv[r] && cv[q]) v = *reinterpret_cast<const float4 *>(x + (((int64_t)n * g.H + (2 * a - 1 + r)) * g.W + (2 * b - 1 + q)) * g.C + c);
            patch[r][q] = v;
        }
    float acc[2][2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) acc[r][q][ch] = 0.f;
#pragma unroll
    for (int wi = 0; wi < 2; ++wi)
#pragma unroll
        for (int wj = 0; wj < 2; ++wj) {
            if (a + wi >= g.Ho || b + wj >= g.Wo) continue;
            const float4 d4 = *reinterpret_cast<const float4 *>(dy + (((int64_t)n * g.Ho + (a + wi)) * g.Wo + (b + wj)) * g.C + c);
            const float d[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) {
                float best = 0.f;
                int bi = -1;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int q = 0; q < 3; ++q) {
                        const int pr = 2 * wi + r, pq = 2 * wj + q;
                        if (!(rv[pr] && cv[pq])) continue;
                        const float4 v4 = patch[pr][pq];
                        const float v = ch == 0 ? v4.x : (ch == 1 ? v4.y : (ch == 2 ? v4.z : v4.w));
                        if (bi < 0 || v > best) { best = v; bi = pr * 5 + pq; }
                    }
                // the block is patch rows/cols 1..2
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        if (bi == (1 + r) * 5 + (1 + q)) acc[r][q][ch] += d[ch];
            }
        }
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (!(rv[1 + r] && cv[1 + q])) continue;
            float4 *o = reinterpret_cast<float4 *>(dx + (((int64_t)n * g.H + (2 * a + r)) * g.W + (2 * b + q)) * g.C + c);
            float4 v = make_float4(acc[r][q][0], acc[r][q][1], acc[r][q][2], acc[r][q][3]);
            if (ACCUM) { const float4 e = *o; v.x += e.x; v.y += e.y; v.z += e.z; v.w += e.w; }
            *o = v;
        }
}

// window == stride, no padding, every extent a multiple of the stride: each input position
// belongs to exactly one window.  One thread per window and V channels.
template <int V, bool ACCUM>
__global__ __launch_bounds__(256) void maxpool_tiled_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dy, float *dx,
                                                                 PoolGeom g, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int CV = g.C / V;
    const int c = (int)(i % CV) * V;
    int64_t t = i / CV;
    const int ow = (int)(t % g.Wo); t /= g.Wo;
    const int oh = (int)(t % g.Ho); t /= g.Ho;
    const int od = (int)(t % g.Do);
    const int n = (int)(t / g.Do);
    float best[V];
    int bi[V];
#pragma unroll
    for (int ch = 0; ch < V; ++ch) { best[ch] = 0.f; bi[ch] = -1; }
    int e = 0;
    for (int p = 0; p < g.kd; ++p)
        for (int q = 0; q < g.kh; ++q)
            for (int r = 0; r < g.kw; ++r, ++e) {
                const float *src = x + ((((int64_t)n * g.D + od * g.sd + p) * g.H + oh * g.sh + q) * g.W + ow * g.sw + r) * g.C + c;
                float v[V];
                if (V == 4) { const float4 v4 = *reinterpret_cast<const float4 *>(src); v[0] = v4.x; v[1 % V] = v4.y; v[2 % V] = v4.z; v[3 % V] = v4.w; }
                else v[0] = *src;
#pragma unroll
                for (int ch = 0; ch < V; ++ch)
                    if (bi[ch] < 0 || v[ch] > best[ch]) { best[ch] = v[ch]; bi[ch] = e; }
            }
    float d[V];
    {
        const float *src = dy + i / CV * g.C + c;
        if (V == 4) { const float4 v4 = *reinterpret_cast<const float4 *>(src); d[0] = v4.x; d[1 % V] = v4.y; d[2 % V] = v4.z; d[3 % V] = v4.w; }
        else d[0] = *src;
    }
    e = 0;
    for (int p = 0; p < g.kd; ++p)
        for (int q = 0; q < g.kh; ++q)
            for (int r = 0; r < g.kw; ++r, ++e) {
                float *dst = dx + ((((int64_t)n * g.D + od * g.sd + p) * g.H + oh * g.sh + q) * g.W + ow * g.sw + r) * g.C + c;
                float o[V];
#pragma unroll
                for (int ch = 0; ch < V; ++ch) o[ch] = bi[ch] == e ? d[ch] : 0.f;
                if (V == 4) {
                    float4 v = make_float4(o[0], o[1 % V], o[2 % V], o[3 % V]);
                    if (ACCUM) { const float4 old = *reinterpret_cast<float4 *>(dst); v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w; }
                    *reinterpret_cast<float4 *>(dst) = v;
                } else {
                    *dst = ACCUM ? *dst + o[0] : o[0];
                }
            }
}

// y[n][c] = (1/S) sum_s x[n][s][c].  One block per (image, 64 channels): its wavefronts -- sixteen for maps of 256 positions
// or more, else four -- take every sixteenth (fourth) position each (ascending, four loads in flight), and the partial sums
// are added in ascending order.
// (With four wavefronts and one load in flight a single volume's 12^3 x 512 map took 0.17 ms: eight blocks, each a chain
// of 432 dependent loads.)
template <int GAP_WAVES>
__global__ __launch_bounds__(64 * GAP_WAVES) void gavgpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, int N, int64_t S, int C)
{
    __shared__ float part[GAP_WAVES][64];
    const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
    const int cblocks = (C + 63) / 64;
    const int64_t n = blockIdx.x / cblocks;
    const int c = (int)(blockIdx.x % cblocks) * 64 + lane;
    float s = 0.f;
    if (c < C) {
        const float *p = x + n * S * C + c;
        int64_t k = w;
        for (; k + 3 * GAP_WAVES < S; k += 4 * GAP_WAVES) {
            const float v0 = p[k * C], v1 = p[(k + GAP_WAVES) * C], v2 = p[(k + 2 * GAP_WAVES) * C], v3 = p[(k + 3 * GAP_WAVES) * C];
            s += v0; s += v1; s += v2; s += v3;
        }
        for (; k < S; k += GAP_WAVES) s += p[k * C];
    }
    part[w][lane] = s;
    __syncthreads();
    if (w == 0 && c < C) {
        float t = part[0][lane];
#pragma unroll
        for (int j = 1; j < GAP_WAVES; ++j) t += part[j][lane];
        y[n * C + c] = t / (float)S;
    }
}

template <bool ACCUM>
__global__ __launch_bounds__(256) void gavgpool_bwd_kernel(const float *__restrict__ dy, float *dx, int N, int64_t S, int C, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % C);
    const int64_t n = i / ((int64_t)S * C);
    const float v = dy[n * C + c] / (float)S;
    dx[i] = ACCUM ? dx[i] + v : v;
}

__global__ __launch_bounds__(256) void bias_add_kernel(float *y, const float *__restrict__ b, int64_t total, int O)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) y[i] += b[i % O];
}

// db[o] = sum_n dy[n][o], n ascending
__global__ __launch_bounds__(256) void bias_grad_kernel(const float *__restrict__ dy, float *__restrict__ db, int N, int O)
{
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= O) return;
    float s = 0.f;
    for (int n = 0; n < N; ++n) s += dy[(int64_t)n * O + o];
    db[o] = s;
}

__device__ __forceinline__ float block_reduce(float v, float *sh, bool is_max)
{
    // 256 threads: wavefront shuffle tree, then the 4 wave results combined in order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_down(v, off, 64);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float r = sh[0];
    for (int w = 1; w < (int)(blockDim.x / 64); ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
    return r;
}

// Softmax cross-entropy of one sample (one block per sample), evaluated so that no digits cancel when the
// sample is classified with a large margin.  With mx the row maximum,
//     -log softmax(z)[t] = (mx - z_t) + log(sum_j exp(z_j - mx)).
// The sum always holds the maximal element's own term exp(0) = 1, so it is taken as 1 + rest, where
// rest = sum over the elements below the maximum of exp(z_j - mx) + (number of maximal elements - 1), and the
// logarithm as log1p(rest): both addends of the loss are non-negative and each is accurate to fp32 rounding,
// where max + log(sum) - z_t loses everything below 1e-7 * |z_t|.
struct RowSums {
    float mx;     // row maximum
    float rest;   // sum_j exp(z_j - mx) without one maximal element's term
};

__device__ __forceinline__ RowSums row_sums(const float *__restrict__ zr, int K, float *sh)
{
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < K; j += blockDim.x) mx = fmaxf(mx, zr[j]);
    mx = block_reduce(mx, sh, true);
    float below = 0.f, ties = 0.f;   // ties: a count, exact in fp32 (K < 2^24 is checked on the host)
    for (int j = threadIdx.x; j < K; j += blockDim.x) {
        const float v = zr[j];
        if (v < mx) below += expf(v - mx);
        else ties += 1.f;
    }
    below = block_reduce(below, sh, false);
    ties = block_reduce(ties, sh, false);
    return RowSums{mx, below + (ties - 1.f)};
}

__global__ __launch_bounds__(256) void softmax_ce_row_kernel(const float *__restrict__ z, const int32_t *__restrict__ labels,
                                                              float *__restrict__ per_sample, int K)
{
    __shared__ float sh[4];
    const int n = blockIdx.x;
    const float *zr = z + (int64_t)n * K;
    const RowSums rs = row_sums(zr, K, sh);
    if (threadIdx.x == 0) {
        const int t = labels[n];
        per_sample[n] = (t >= 0 && t < K) ? (rs.mx - zr[t]) + log1pf(rs.rest) : 0.f;
    }
}

__global__ __launch_bounds__(64) void loss_mean_kernel(const float *__restrict__ per_sample, float *__restrict__ loss, int N)
{
    double s = 0.0;
    for (int n = threadIdx.x; n < N; n += 64) s += (double)per_sample[n];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
    if (threadIdx.x == 0) loss[0] = (float)(s / (double)N);
}

// dz_j = (softmax(z)_j - [j == t]) / N.  For the labelled class softmax - 1 = -(sum of the other classes' terms) /
// (sum of all terms): the numerator is summed without the labelled class's own term instead of being formed as a
// difference from 1, so a confidently classified sample keeps a gradient accurate to rounding (p_t - 1 in fp32 would be 0
// or a few bits).
template <bool ACCUM>
__global__ __launch_bounds__(256) void softmax_ce_bwd_kernel(const float *__restrict__ z, const int32_t *__restrict__ labels,
                                                              float *dz, int K, float inv_n)
{
    __shared__ float sh[4];
    const int n = blockIdx.x;
    const float *zr = z + (int64_t)n * K;
    const int t = labels[n];
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < K; j += blockDim.x) mx = fmaxf(mx, zr[j]);
    mx = block_reduce(mx, sh, true);
    float others = 0.f;
    for (int j = threadIdx.x; j < K; j += blockDim.x)
        if (j != t) others += expf(zr[j] - mx);
    others = block_reduce(others, sh, false);
    const float et = (t >= 0 && t < K) ? expf(zr[t] - mx) : 0.f;
    const float scale = inv_n / (others + et);
    for (int j = threadIdx.x; j < K; j += blockDim.x) {
        const float v = (j == t ? -others : expf(zr[j] - mx)) * scale;
        float *o = dz + (int64_t)n * K + j;
        *o = ACCUM ? *o + v : v;
    }
}

bool pool_ok(const PoolGeom &g)
{
    if (g.N <= 0 || g.C <= 0 || g.D <= 0 || g.H <= 0 || g.W <= 0) return false;
    if (g.kd <= 0 || g.kh <= 0 || g.kw <= 0 || g.sd <= 0 || g.sh <= 0 || g.sw <= 0 || g.pd < 0 || g.ph < 0 || g.pw < 0) return false;
    if (g.Do != (g.D + 2 * g.pd - g.kd) / g.sd + 1 || g.Ho != (g.H + 2 * g.ph - g.kh) / g.sh + 1 ||
        g.Wo != (g.W + 2 * g.pw - g.kw) / g.sw + 1)
        return false;
    return g.Do > 0 && g.Ho > 0 && g.Wo > 0;
}

inline dim3 blocks_for(int64_t total) { return dim3((unsigned)((total + 255) / 256)); }
// an eighth of the workgroups of a launch whose index space is split over the XCDs (pool_block); 0: plain order
inline unsigned pool_spread(int64_t total)
{
    static const bool off = getenv("POOCH_NO_POOL_XCD") != nullptr;
    const int64_t blocks = (total + 255) / 256;
    return (off || blocks < 64) ? 0u : (unsigned)((blocks + 7) / 8);
}

}  // namespace

hipError_t maxpool_fwd(const float *x, float *y, const PoolGeom &g, hipStream_t s)
{
    if (!x || !y || !pool_ok(g)) return hipErrorInvalidValue;
    const int64_t total = (int64_t)g.N * g.Do * g.Ho * g.Wo * g.C;
    if (g.C % 4 == 0 && ((uintptr_t)x | (uintptr_t)y) % 16 == 0) {
        const unsigned sp = pool_spread(total / 4);
        maxpool_fwd_vec4_kernel<<<sp ? dim3(8 * sp) : blocks_for(total / 4), dim3(256), 0, s>>>(x, y, g, total / 4, sp);
    } else {
        maxpool_fwd_kernel<<<blocks_for(total), dim3(256), 0, s>>>(x, y, g, total);
    }
    return hipGetLastError();
}

hipError_t maxpool_bwd(const float *x, const float *dy, float *dx, const PoolGeom &g, bool accumulate, hipStream_t s)
{
    if (!x || !dy || !dx || !pool_ok(g)) return hipErrorInvalidValue;
    const bool al16 = ((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx) % 16 == 0;
    if (g.D == 1 && g.kd == 1 && g.sd == 1 && g.pd == 0 && g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2 && g.ph == 1 && g.pw == 1 &&
        g.C % 4 == 0 && al16) {
        const int HB = (g.H + 1) / 2, WB = (g.W + 1) / 2;
        const int64_t tot = (int64_t)g.N * HB * WB * (g.C / 4);
        const unsigned sp = pool_spread(tot);
        const dim3 grid = sp ? dim3(8 * sp) : blocks_for(tot);
        if (accumulate) maxpool_k3s2p1_bwd_kernel<true><<<grid, dim3(256), 0, s>>>(x, dy, dx, g, HB, WB, tot, sp);
        else maxpool_k3s2p1_bwd_kernel<false><<<grid, dim3(256), 0, s>>>(x, dy, dx, g, HB, WB, tot, sp);
        return hipGetLastError();
    }
    if (g.kd == g.sd && g.kh == g.sh && g.kw == g.sw && g.pd == 0 && g.ph == 0 && g.pw == 0 && g.D % g.sd == 0 && g.H % g.sh == 0 &&
        g.W % g.sw == 0) {
        const bool v4 = g.C % 4 == 0 && al16;
        const int64_t tot = (int64_t)g.N * g.Do * g.Ho * g.Wo * (g.C / (v4 ? 4 : 1));
#define TILED(V, A) maxpool_tiled_bwd_kernel<V, A><<<blocks_for(tot), dim3(256), 0, s>>>(x, dy, dx, g, tot)
        if (v4) { if (accumulate) TILED(4, true); else TILED(4, false); }
        else { if (accumulate) TILED(1, true); else TILED(1, false); }
#undef TILED
        return hipGetLastError();
    }
    const int64_t total = (int64_t)g.N * g.D * g.H * g.W * g.C;
    if (accumulate) maxpool_bwd_kernel<true><<<blocks_for(total), dim3(256), 0, s>>>(x, dy, dx, g, total);
    else maxpool_bwd_kernel<false><<<blocks_for(total), dim3(256), 0, s>>>(x, dy, dx, g, total);
    return hipGetLastError();
}

hipError_t gavgpool_fwd(const float *x, float *y, int N, int64_t S, int C, hipStream_t s)
{
    if (!x || !y || N <= 0 || S <= 0 || C <= 0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((int64_t)N * ((C + 63) / 64)));
    if (S >= 256) gavgpool_fwd_kernel<16><<<grid, dim3(1024), 0, s>>>(x, y, N, S, C);
    else gavgpool_fwd_kernel<4><<<grid, dim3(256), 0, s>>>(x, y, N, S, C);
    return hipGetLastError();
}

hipError_t gavgpool_bwd(const float *dy, float *dx, int N, int64_t S, int C, bool accumulate, hipStream_t s)
{
    if (!dy || !dx || N <= 0 || S <= 0 || C <= 0) return hipErrorInvalidValue;
    const int64_t total = (int64_t)N * S * C;
    if (accumulate) gavgpool_bwd_kernel<true><<<blocks_for(total), dim3(256), 0, s>>>(dy, dx, N, S, C, total);
    else gavgpool_bwd_kernel<false><<<blocks_for(total), dim3(256), 0, s>>>(dy, dx, N, S, C, total);
    return hipGetLastError();
}

hipError_t bias_add(float *y, const float *b, int N, int O, hipStream_t s)
{
    if (!y || !b || N <= 0 || O <= 0) return hipErrorInvalidValue;
    const int64_t total = (int64_t)N * O;
    bias_add_kernel<<<blocks_for(total), dim3(256), 0, s>>>(y, b, total, O);
    return hipGetLastError();
}

hipError_t bias_grad(const float *dy, float *db, int N, int O, hipStream_t s)
{
    if (!dy || !db || N <= 0 || O <= 0) return hipErrorInvalidValue;
    bias_grad_kernel<<<blocks_for(O), dim3(256), 0, s>>>(dy, db, N, O);
    return hipGetLastError();
}

hipError_t softmax_ce_fwd(const float *z, const int32_t *labels, float *per_sample, float *loss, int N, int K, hipStream_t s)
{
    if (!z || !labels || !per_sample || !loss || N <= 0 || K <= 0 || K >= (1 << 24)) return hipErrorInvalidValue;
    softmax_ce_row_kernel<<<dim3(N), dim3(256), 0, s>>>(z, labels, per_sample, K);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    loss_mean_kernel<<<dim3(1), dim3(64), 0, s>>>(per_sample, loss, N);
    return hipGetLastError();
}

hipError_t softmax_ce_bwd(const float *z, const int32_t *labels, float *dz, int N, int K, bool accumulate, hipStream_t s)
{
    if (!z || !labels || !dz || N <= 0 || K <= 0 || K >= (1 << 24)) return hipErrorInvalidValue;
    const float inv_n = 1.f / (float)N;
    if (accumulate) softmax_ce_bwd_kernel<true><<<dim3(N), dim3(256), 0, s>>>(z, labels, dz, K, inv_n);
    else softmax_ce_bwd_kernel<false><<<dim3(N), dim3(256), 0, s>>>(z, labels, dz, K, inv_n);
    return hipGetLastError();
}

}  // namespace pk
