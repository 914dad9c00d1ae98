// fp32 MFMA implicit-GEMM convolution for gfx950: forward, data gradient, filter gradient.
//
// The paper (section 3.3) only says that convolution layers carry "large computation
// complexity" and are what hides swap traffic; it uses a vendor library for them.  Here
// they are written for CDNA4: channels-last tensors make every GEMM operand row a run of
// contiguous channels, tiles are staged through LDS with 16-byte loads/stores, and each
// 64-lane wavefront owns a TM x TN grid of 32x32 accumulators fed by
// v_mfma_f32_32x32x2_f32.  No atomics: the filter gradient's long reduction is split over
// workgroups into a workspace and summed in a fixed order.
// Beside the general kernels (igemm_kernel: forward and data gradient; wgrad_kernel: filter
// gradient) there are kernels for the shapes on which those fall short: wgrad_halo_kernel (3-wide
// filters on 32 or 64 channels: the taps share what is staged), and for 3 x 3 x 3 filters on volumes
// of whole 2 x 8 x 8 bricks conv3_halo_kernel (32 -> 32 channels), wgrad3_brick_kernel (any multiple
// of 32 channels) and conv3_c1_kernel / wgrad3_c1_kernel (a network input with one live channel),
// which keep a brick of the input with its halo in LDS for all 27 taps; wgrad2_brick_kernel does the
// same for 3 x 3 filters on images of whole 8 x 8 bricks, and stem7_fwd_kernel / stem7_wgrad_kernel
// serve the 7 x 7 stride-2 first layer of ResNet.
#include "kernels.h"

#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <type_traits>

namespace pk {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BK = 16;   // reduction slice per main-loop iteration
constexpr int LDK = 20;  // LDS row stride (floats) of [row][k] tiles: 16-byte rows, conflict-free b128 reads
constexpr int NXCD = 8;
constexpr int NCU = 256;  // compute units of the one GPU this library is written for

// Loads of tensor data name the global address space.  A pointer that comes out of a parameter
// struct is a generic one to the compiler, and a generic ("flat") load is also counted by the
// counter LDS reads are waited on: the wait before a slice's first MFMA would then sit out the
// whole latency of the prefetch issued just before it.
typedef const __attribute__((address_space(1))) f32x4 *gvec4_ptr;
typedef const __attribute__((address_space(1))) float *gfloat_ptr;
__device__ __forceinline__ f32x4 ldg4(const float *p) { return *(gvec4_ptr)(p); }
__device__ __forceinline__ float ldg1(const float *p) { return *(gfloat_ptr)(p); }

// 16 zero bytes every kernel may read: elements that do not exist (padding, rows or slices past
// the end) are loaded from here instead of being branched around or masked afterwards
__device__ __attribute__((aligned(16))) const float g_zero4[4] = {0.f, 0.f, 0.f, 0.f};

struct IGemmP {
    const float *src;  // forward: x; data gradient: dy (channels-last)
    const float *wgt;  // [Nout][Kred]
    float *dst;        // [M][Nout]
    float *stats;      // STATS kernels: per row tile, mean[Nout] then M2[Nout] of the tile's rows of dst
    int M, Nout, Kred, Cs;
    int Dr, Hr, Wr;  // spatial dims the GEMM rows enumerate
    int Ds, Hs, Ws;  // spatial dims of src
    int kd, kh, kw, sd, sh, sw, pd, ph, pw;
    int tiles_n, total_tiles, chunk;
    // split over the reduction: ksplit > 1 gives workgroup (tile, ks) the slices [ks * kslices, (ks + 1) * kslices) and sends its
    // result to dst + ks * M * Nout (a stack of partial results that splitk_reduce_kernel sums in a fixed order)
    int ksplit, kslices;
    // destination rows: identity, or (dst_strided) GEMM row (n,d,h,w) -> row ((n*DD + d*SD)*HD + h*SH)*WD + w*SW
    int dst_strided, DD, HD, WD, SD, SH, SW;
    // bd > 0: the rows of a tile are a brick of bd x 8 x 8 positions (d, h, w) instead of consecutive rows; tiles enumerate the
    // bricks of (n, d, h, w) with w fastest.  Requires bd * 64 == rows per tile and Dr % bd == Hr % 8 == Wr % 8 == 0.
    int bd;
    // > 0: only the first `live` of the Cs source channels can be non-zero, in src and in wgt (forward of a padded network input)
    int live;
};

// coordinate in the source tensor touched by filter tap `a` for a row whose base is `base`
template <bool DGRAD>
__device__ __forceinline__ bool src_coord(int base, int a, int s, int S, int &q)
{
    if (!DGRAD) {
        q = base + a;
        return (unsigned)q < (unsigned)S;
    } else {
        // q*s == base - a must hold exactly; no branches so that callers stay straight-line
        const int t = base - a;
        const int tt = t < 0 ? 0 : t;
        q = s == 1 ? tt : tt / s;
        return (t >= 0) & (q * s == tt) & (q < S);
    }
}

// XCD-aware tile order: hardware deals consecutive workgroup ids round-robin to the 8
// XCDs; give each XCD a contiguous range of tiles so that neighbours share its L2.
__device__ __forceinline__ int remap_tile(int wg, int chunk) { return (wg % NXCD) * chunk + wg / NXCD; }

// Four waves of four accumulator blocks: the compiler is asked for four waves per SIMD (128 registers, accumulators included).
// Left alone it gave the accumulating instantiations 142 and the 256 x 64 tile's 130, which cost them the fourth workgroup
// of a compute unit (1 x 1 256 -> 64 data gradient at batch 640: 1.00 -> 0.91 ms; 3 x 3 64 -> 64 forward 1.32 -> 1.29).
// Not asked of the 256 x 64 tile's per-thread-tap and general address paths, which would spill 8 - 14 registers.
template <int WGM, int WGN, int TM, int TN, int BKT, bool VEC, int LIN, bool DGRAD, bool ACCUM, bool STATS = false>
__global__ __launch_bounds__(64 * WGM * WGN, (TM * TN == 4 && BKT == 16 && WGM * WGN == 4 && (WGM == 2 || LIN == 1 || LIN == 3)) ? 4 : 1)
void igemm_kernel(IGemmP p)
{
    // BKT = reduction slice per main-loop iteration; LDS rows are BKT + 4 floats apart (16-byte
    // aligned, conflict-free 128-bit reads)
    constexpr int NT = 64 * WGM * WGN;
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int LDT = BKT + 4;
    constexpr int KQ = BKT / 4;                      // float4 per tile row
    constexpr int RPP = NT / KQ;                     // rows covered per pass of vector loads
    constexpr int A_V = (BM + RPP - 1) / RPP, B_V = (BN + RPP - 1) / RPP;
    constexpr int RPS = NT / BKT;                    // rows per pass of scalar loads
    constexpr int A_S = BM / RPS, B_S = BN / RPS;
    static_assert(NT % KQ == 0 && NT % BKT == 0 && BM % RPS == 0 && BN % RPS == 0, "tile/threads mismatch");

    // operand tiles during the main loop; afterwards the same memory stages each wavefront's
    // 32 x (TN*32) accumulator blocks on their way out (row stride CST floats)
    constexpr int CST = TN * 32 + 4;
    constexpr int SM_AB = (BM + BN) * LDT, SM_C = WGM * WGN * 32 * CST;
    __shared__ __attribute__((aligned(16))) float smem[SM_AB > SM_C ? SM_AB : SM_C];
    float *const As = smem;
    float *const Bs = smem + BM * LDT;
    __shared__ int4 rowinfo[BM];
    __shared__ int rowdst[BM];

    const int tid = threadIdx.x;
    const int logical_wg = remap_tile(blockIdx.x, p.chunk);
    if (logical_wg >= p.total_tiles * p.ksplit) return;
    const int ks = logical_wg / p.total_tiles, logical = logical_wg % p.total_tiles;
    const int m0 = (logical / p.tiles_n) * BM, n0 = (logical % p.tiles_n) * BN;
    float *const dst = p.dst + (int64_t)ks * p.M * p.Nout;

    for (int r = tid; r < BM; r += NT) {
        int m = m0 + r;
        int4 ri = make_int4(-1, 0, 0, 0);
        int rd = -1;
        if (m < p.M) {
            int n, d_, h_, w_;
            if (p.bd > 0) {
                // Under a filter with depth, BM consecutive rows (a strip of one or two lines) touch nine times their own
                // input; a brick touches (bd + 2) * 10 * 10 / (bd * 64) of it (2.3 for bd = 4), whatever the caches hold.
                int t = m0 / BM;
                const int nbw = p.Wr / 8, nbh = p.Hr / 8, nbd = p.Dr / p.bd;
                w_ = (t % nbw) * 8 + r % 8;
                t /= nbw;
                h_ = (t % nbh) * 8 + (r / 8) % 8;
                t /= nbh;
                d_ = (t % nbd) * p.bd + r / 64;
                n = t / nbd;
                m = ((n * p.Dr + d_) * p.Hr + h_) * p.Wr + w_;
            } else {
                w_ = m % p.Wr;
                int t = m / p.Wr;
                h_ = t % p.Hr;
                t /= p.Hr;
                d_ = t % p.Dr;
                n = t / p.Dr;
            }
            ri = DGRAD ? make_int4(n, d_ + p.pd, h_ + p.ph, w_ + p.pw)
                       : make_int4(n, d_ * p.sd - p.pd, h_ * p.sh - p.ph, w_ * p.sw - p.pw);
            rd = p.dst_strided ? ((n * p.DD + d_ * p.SD) * p.HD + h_ * p.SH) * p.WD + w_ * p.SW : m;
        }
        rowinfo[r] = ri;
        rowdst[r] = rd;
    }
    __syncthreads();

    f32x4 av[VEC ? A_V : 1], bv[VEC ? B_V : 1];
    float as[VEC ? 1 : A_S], bs[VEC ? 1 : B_S];
    int4 ri_reg[VEC ? A_V : 1];
    unsigned amask = 0, bmask = 0;                   // vector path: which prefetched float4 hold real data
    const int vrow = tid / KQ, vk = 4 * (tid % KQ);  // vector path: this thread's row within a pass, k offset
    if (VEC) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            ri_reg[i] = rowinfo[(vrow + i * RPP) % BM];
            if (vrow + i * RPP >= BM) ri_reg[i].x = -1;
        }
    }
    // when every filter tap spans a whole number of slices, the tap of a slice is the same for
    // all threads: its decomposition then runs on the scalar unit
    const bool tap_uniform = p.Cs % BKT == 0;

    // LIN (requires Cs % BKT == 0, and unit strides for the data gradient): the source element of
    // row i at the current slice is abase[i] + delta, where delta depends only on the slice (scalar
    // unit) and abase[i] is fixed for the tile.  Per slice and row that leaves three coordinate
    // range checks and one 64-bit add on the vector unit -- no multiplies, no divisions.
    // LIN == 2 (forward only; Cs divides BKT, e.g. a 4-channel first layer): a slice spans BKT / Cs
    // taps, so the tap belongs to the thread (it is fixed by the thread's k offset) and advances by
    // BKT / Cs per slice with carries -- still no divisions after the set-up.
    int64_t abase[LIN ? A_V : 1];
    const float *bptr[LIN ? B_V : 1];
    bool brow[LIN ? B_V : 1];
    int ta = 0, tb = 0, te = 0, tc = 0;              // tap (a, b, e) and channel offset of the slice start
    int pk = vk;                                     // LIN == 2: this thread's position in the reduction
    const int nk_all = (p.Kred + BKT - 1) / BKT;
    const int it_beg = ks * p.kslices, it_end = p.ksplit > 1 ? min(nk_all, it_beg + p.kslices) : nk_all;
    // LIN == 1 walks the reduction channel slice by channel slice and, inside a slice, tap by tap (the sum's terms are the
    // same, their order is this path's own): consecutive steps then read the same channels of pixels one tap apart --
    // what a neighbouring row of the tile read a step earlier -- so the input is fetched into the XCD's L2 about once
    // instead of once per tap, the taps of one slice being many steps apart otherwise.
    const int ntaps = p.kd * p.kh * p.kw;
    int koff = 0;                                    // offset of the step's filter slice inside a filter row: tap * Cs + tc
    if (LIN == 1 && it_beg > 0) {                    // a later part of the reduction: its first step's slice and tap
        const int tap = it_beg % ntaps;
        tc = (it_beg / ntaps) * BKT;
        te = tap % p.kw;
        tb = (tap / p.kw) % p.kh;
        ta = tap / (p.kw * p.kh);
        koff = tap * p.Cs + tc;
    }
    if (LIN == 2) {
        const int tap = vk / p.Cs;
        te = tap % p.kw;
        tb = (tap / p.kw) % p.kh;
        ta = tap / (p.kw * p.kh);
    }
    // LIN == 3 (one tap, no padding: a plain GEMM whose A rows are pixels): every row that exists is valid at every step, so
    // the loop keeps one pointer per row and adds BKT to it -- no range checks, no selects.  Rows past the end of either
    // operand alias the tile's first row: what they produce is never stored.
    const float *aptr[LIN == 3 ? A_V : 1];
    if (LIN == 3) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            const int4 ri = ri_reg[i].x >= 0 ? ri_reg[i] : rowinfo[0];
            aptr[i] = p.src + (((((int64_t)ri.x * p.Ds + ri.y) * p.Hs + ri.z) * p.Ws + ri.w) * p.Cs + vk + (int64_t)it_beg * BKT);
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            int n = n0 + vrow + i * RPP;
            if (vrow + i * RPP >= BN || n >= p.Nout) n = n0;
            bptr[i] = p.wgt + ((int64_t)n * p.Kred + vk + (int64_t)it_beg * BKT);
        }
    } else if (LIN) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            const int4 ri = ri_reg[i];
            abase[i] = ((((int64_t)ri.x * p.Ds + ri.y) * p.Hs + ri.z) * p.Ws + ri.w) * p.Cs + (LIN == 2 ? vk % p.Cs : vk);
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            const int n = n0 + vrow + i * RPP;
            brow[i] = (vrow + i * RPP < BN) & (n < p.Nout);
            bptr[i] = p.wgt + (brow[i] ? (int64_t)n * p.Kred + vk : 0);
        }
    }
    auto load_tiles_gemm = [&]() {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            av[i] = ldg4(aptr[i]);
            aptr[i] += BKT;
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            bv[i] = ldg4(bptr[i]);
            bptr[i] += BKT;
        }
    };
    auto load_tiles_tap = [&](bool live) {
        const bool kok = live & (pk < p.Kred);
        const int64_t tapoff = (((int64_t)ta * p.Hs + tb) * p.Ws + te) * p.Cs;
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            const int4 ri = ri_reg[i];
            const bool ok = kok & (ri.x >= 0) & ((unsigned)(ri.y + ta) < (unsigned)p.Ds) & ((unsigned)(ri.z + tb) < (unsigned)p.Hs) &
                            ((unsigned)(ri.w + te) < (unsigned)p.Ws);
            av[i] = ldg4(ok ? p.src + (abase[i] + tapoff) : g_zero4);
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            const bool ok = kok & brow[i];
            bv[i] = ldg4(ok ? bptr[i] : g_zero4);
            bptr[i] += BKT;
        }
        pk += BKT;
        te += BKT / p.Cs;
        while (te >= p.kw) {
            te -= p.kw;
            if (++tb == p.kh) {
                tb = 0;
                ++ta;
            }
        }
    };
    auto load_tiles_lin = [&](bool live) {
        const int64_t tapoff = (((int64_t)ta * p.Hs + tb) * p.Ws + te) * p.Cs;
        const int64_t delta = (DGRAD ? -tapoff : tapoff) + tc;
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            const int4 ri = ri_reg[i];
            const int qd = DGRAD ? ri.y - ta : ri.y + ta;
            const int qh = DGRAD ? ri.z - tb : ri.z + tb;
            const int qw = DGRAD ? ri.w - te : ri.w + te;
            const bool ok = live & (ri.x >= 0) & ((unsigned)qd < (unsigned)p.Ds) & ((unsigned)qh < (unsigned)p.Hs) &
                            ((unsigned)qw < (unsigned)p.Ws);
            av[i] = ldg4(ok ? p.src + (abase[i] + delta) : g_zero4);
        }
        amask = ~0u;
        bmask = ~0u;
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            const bool ok = live & brow[i];
            bv[i] = ldg4(ok ? bptr[i] + koff : g_zero4);
        }
        // next step: the next tap of this channel slice, or the first tap of the next slice
        koff += p.Cs;
        if (++te == p.kw) {
            te = 0;
            if (++tb == p.kh) {
                tb = 0;
                if (++ta == p.kd) {
                    ta = 0;
                    tc += BKT;
                    koff = tc;
                }
            }
        }
    };

    // The vector path is branch-free on purpose: addresses of elements that do not exist are
    // clamped to offset 0 (always readable) and the value is zeroed when it is stored to LDS.
    // Straight-line code lets the scheduler spread this address arithmetic and the loads
    // between the MFMAs of the slice being multiplied, instead of running them as a separate phase.
    auto load_tiles = [&](int k0) {
        if (VEC) {
            const int k = k0 + vk;
            const bool kok = k < p.Kred;
            int tap, c;
            if (tap_uniform) {
                tap = k0 / p.Cs;
                c = k0 - tap * p.Cs + vk;
            } else {
                const int kc = kok ? k : 0;
                tap = kc / p.Cs;
                c = kc - tap * p.Cs;
            }
            const int e = tap % p.kw;
            const int t2 = tap / p.kw;
            const int b = t2 % p.kh;
            const int a = t2 / p.kh;
            amask = 0;
#pragma unroll
            for (int i = 0; i < A_V; ++i) {
                const int4 ri = ri_reg[i];
                int qd, qh, qw;
                const bool vd = src_coord<DGRAD>(ri.y, a, p.sd, p.Ds, qd);
                const bool vh = src_coord<DGRAD>(ri.z, b, p.sh, p.Hs, qh);
                const bool vw = src_coord<DGRAD>(ri.w, e, p.sw, p.Ws, qw);
                const bool ok = kok & (ri.x >= 0) & vd & vh & vw;
                const int64_t off = ((((int64_t)ri.x * p.Ds + qd) * p.Hs + qh) * p.Ws + qw) * p.Cs + c;
                av[i] = ldg4(p.src + (ok ? off : 0));
                amask |= (ok ? 1u : 0u) << i;
            }
            bmask = 0;
#pragma unroll
            for (int i = 0; i < B_V; ++i) {
                const int n = n0 + vrow + i * RPP;
                const bool ok = kok & (vrow + i * RPP < BN) & (n < p.Nout);
                bv[i] = ldg4(p.wgt + (ok ? (int64_t)n * p.Kred + k : 0));
                bmask |= (ok ? 1u : 0u) << i;
            }
        } else {
            const int k = k0 + (tid % BKT);
            const bool kok = k < p.Kred;
            int a = 0, b = 0, e = 0, c = 0;
            if (kok) {
                const int tap = k / p.Cs;
                c = k - tap * p.Cs;
                e = tap % p.kw;
                const int t2 = tap / p.kw;
                b = t2 % p.kh;
                a = t2 / p.kh;
            }
#pragma unroll
            for (int i = 0; i < A_S; ++i) {
                float v = 0.f;
                const int4 ri = rowinfo[tid / BKT + i * RPS];
                int qd, qh, qw;
                if (kok && ri.x >= 0 && src_coord<DGRAD>(ri.y, a, p.sd, p.Ds, qd) &&
                    src_coord<DGRAD>(ri.z, b, p.sh, p.Hs, qh) && src_coord<DGRAD>(ri.w, e, p.sw, p.Ws, qw)) {
                    const int64_t off = ((((int64_t)ri.x * p.Ds + qd) * p.Hs + qh) * p.Ws + qw) * p.Cs + c;
                    v = ldg1(p.src + off);
                }
                as[i] = v;
            }
#pragma unroll
            for (int i = 0; i < B_S; ++i) {
                const int n = n0 + tid / BKT + i * RPS;
                bs[i] = (kok && n < p.Nout) ? ldg1(p.wgt + ((int64_t)n * p.Kred + k)) : 0.f;
            }
        }
    };

    auto store_tiles = [&]() {
        if (VEC) {
#pragma unroll
            for (int i = 0; i < A_V; ++i)
                if (vrow + i * RPP < BM)
                    *reinterpret_cast<f32x4 *>(&As[(vrow + i * RPP) * LDT + vk]) = (LIN || ((amask >> i) & 1u)) ? av[i] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < B_V; ++i)
                if (vrow + i * RPP < BN)
                    *reinterpret_cast<f32x4 *>(&Bs[(vrow + i * RPP) * LDT + vk]) = (LIN || ((bmask >> i) & 1u)) ? bv[i] : f32x4{0.f, 0.f, 0.f, 0.f};
        } else {
#pragma unroll
            for (int i = 0; i < A_S; ++i) As[(tid / BKT + i * RPS) * LDT + (tid % BKT)] = as[i];
#pragma unroll
            for (int i = 0; i < B_S; ++i) Bs[(tid / BKT + i * RPS) * LDT + (tid % BKT)] = bs[i];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int lane = tid % 64, wave = tid / 64;
    const int wm = wave / WGN, wn = wave % WGN;
    const int r = lane % 32, h = lane / 32;

    const int nk = it_end;
    if (LIN == 3) {
        if (it_beg < nk) load_tiles_gemm();
    } else if (LIN == 2) load_tiles_tap(true);
    else if (LIN) load_tiles_lin(it_beg < nk);
    else load_tiles(it_beg * BKT);
    for (int it = it_beg; it < nk; ++it) {
        store_tiles();
        __syncthreads();
        if (LIN == 3) {
            if (it + 1 < nk) load_tiles_gemm();       // uniform branch: nothing is read past the end of a row
        } else if (LIN == 2) load_tiles_tap(it + 1 < nk);
        else if (LIN) load_tiles_lin(it + 1 < nk);     // past the end: every element is masked off
        else if (VEC) load_tiles((it + 1) * BKT);
        else if (it + 1 < nk) load_tiles((it + 1) * BKT);

        // per 16-wide sub-slice s: lane half h covers k = 16s + 8h .. 16s + 8h + 7; MFMA step t multiplies k = 16s + 8h + t
#pragma unroll
        for (int sub = 0; sub < BKT / 16; ++sub) {
            float af[TM][8], bf[TN][8];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float *ap = &As[(wm * TM * 32 + i * 32 + r) * LDT + sub * 16 + h * 8];
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(ap);
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(ap + 4);
                af[i][0] = lo.x; af[i][1] = lo.y; af[i][2] = lo.z; af[i][3] = lo.w;
                af[i][4] = hi.x; af[i][5] = hi.y; af[i][6] = hi.z; af[i][7] = hi.w;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float *bp = &Bs[(wn * TN * 32 + j * 32 + r) * LDT + sub * 16 + h * 8];
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(bp);
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(bp + 4);
                bf[j][0] = lo.x; bf[j][1] = lo.y; bf[j][2] = lo.z; bf[j][3] = lo.w;
                bf[j][4] = hi.x; bf[j][5] = hi.y; bf[j][6] = hi.z; bf[j][7] = hi.w;
            }
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[j][t], af[i][t], acc[i][j], 0, 0, 0);
            // ask the scheduler for a regular pattern -- one MFMA, then a few address-arithmetic
            // instructions and at most one load of the prefetch -- instead of its own clustering
            // (measured: 120 -> 125 TFLOP/s on the large layers)
#pragma unroll
            for (int q = 0; q < TM * TN * 8; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);   // VALU
                __builtin_amdgcn_sched_group_barrier(0x004, 2, 0);   // SALU
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read
            }
        }
        __syncthreads();
    }

    // The MFMA is issued with the operands swapped (B, A), so each 32x32 block comes out transposed:
    // accumulator element v of a lane belongs to GEMM row r and GEMM column 8*(v/4) + 4*h + v%4.
    // A lane therefore owns runs of four consecutive output channels: 16-byte stores (and loads, when
    // accumulating) instead of four scalar ones.
    const bool vec_out = p.Nout % 4 == 0;
    if (vec_out) {
        // Through LDS, so that a store instruction of the wavefront covers whole rows of its block
        // (TN*128 contiguous bytes each) instead of 32-byte pieces of 32 different rows.
        constexpr int LPR = TN * 8;          // lanes per row, 16 bytes each
        constexpr int RPI = 64 / LPR;        // rows per store instruction
        constexpr int NQ = 32 / RPI;
        float *cw = smem + wave * 32 * CST;
        const int orow = lane / LPR, ocol = 4 * (lane % LPR);
        const int ncol = n0 + wn * TN * 32 + ocol;
        // STATS: count, mean and sum of squared deviations (M2) of this lane's four columns over the
        // rows this wavefront has written so far.  Per 32-row block: mean, then M2 about that mean
        // (no cancellation), merged into the running triple by the pairwise update of Chan et al.
        float rn = 0.f;
        f32x4 rmean = {0.f, 0.f, 0.f, 0.f}, rm2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            // accumulating: the block's old values are all requested here, before the block goes through LDS, without branches
            // (rows that do not exist read the zero page).  Left to the compiler, each row's load sat under that row's branch,
            // right before its store: one memory round trip after the other, NQ per block.
            f32x4 oldv[ACCUM ? NQ : 1];
            if constexpr (ACCUM) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int m = rowdst[wm * TM * 32 + i * 32 + q * RPI + orow];
                    const float *op = (m >= 0 && ncol < p.Nout) ? dst + (int64_t)m * p.Nout + ncol : g_zero4;
                    oldv[q] = __builtin_nontemporal_load((gvec4_ptr)(op));
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 val = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    *reinterpret_cast<f32x4 *>(&cw[r * CST + j * 32 + 8 * g + 4 * h]) = val;
                }
            __syncthreads();
            f32x4 vq[STATS ? NQ : 1];
            bool okq[STATS ? NQ : 1];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int row = q * RPI + orow;
                const int m = rowdst[wm * TM * 32 + i * 32 + row];
                f32x4 val = *reinterpret_cast<const f32x4 *>(&cw[row * CST + ocol]);
                if constexpr (STATS) {
                    vq[q] = val;
                    okq[q] = m >= 0;
                }
                if (m >= 0 && ncol < p.Nout) {
                    f32x4 *dp = reinterpret_cast<f32x4 *>(dst + (int64_t)m * p.Nout + ncol);
                    if constexpr (ACCUM) val = oldv[q] + val;
                    __builtin_nontemporal_store(val, dp);
                }
            }
            if constexpr (STATS) {
                // rows that exist form a prefix of the block
                int nb = p.M - (m0 + (wm * TM + i) * 32);
                nb = nb < 0 ? 0 : (nb > 32 ? 32 : nb);
                if (nb > 0) {   // uniform over the wavefront
                    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        if (okq[q]) sum += vq[q];
#pragma unroll
                    for (int mask = LPR; mask < 64; mask <<= 1) {
                        sum.x += __shfl_xor(sum.x, mask, 64); sum.y += __shfl_xor(sum.y, mask, 64);
                        sum.z += __shfl_xor(sum.z, mask, 64); sum.w += __shfl_xor(sum.w, mask, 64);
                    }
                    const float nbf = (float)nb;
                    const f32x4 mb = sum / nbf;
                    f32x4 d2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        if (okq[q]) {
                            const f32x4 d = vq[q] - mb;
                            d2 += d * d;
                        }
#pragma unroll
                    for (int mask = LPR; mask < 64; mask <<= 1) {
                        d2.x += __shfl_xor(d2.x, mask, 64); d2.y += __shfl_xor(d2.y, mask, 64);
                        d2.z += __shfl_xor(d2.z, mask, 64); d2.w += __shfl_xor(d2.w, mask, 64);
                    }
                    const float tot = rn + nbf;
                    const f32x4 delta = mb - rmean;
                    rmean += delta * (nbf / tot);
                    rm2 += d2 + delta * delta * (rn * nbf / tot);
                    rn = tot;
                }
            }
            if (i + 1 < TM || STATS) __syncthreads();
        }
        if constexpr (STATS) {
            // the wavefronts that share these columns (same wn) are merged in wm order by the first
            float *sm = smem;   // [wave][mean, M2][TN * 32]
            if (orow == 0) {
                *reinterpret_cast<f32x4 *>(&sm[(wave * 2 + 0) * TN * 32 + ocol]) = rmean;
                *reinterpret_cast<f32x4 *>(&sm[(wave * 2 + 1) * TN * 32 + ocol]) = rm2;
            }
            __syncthreads();
            if (wm == 0 && orow == 0 && ncol < p.Nout) {
#pragma unroll
                for (int w2 = 1; w2 < WGM; ++w2) {
                    int nb = p.M - (m0 + w2 * TM * 32);
                    nb = nb < 0 ? 0 : (nb > TM * 32 ? TM * 32 : nb);
                    if (nb > 0) {
                        const int ow = w2 * WGN + wn;
                        const f32x4 mb = *reinterpret_cast<const f32x4 *>(&sm[(ow * 2 + 0) * TN * 32 + ocol]);
                        const f32x4 d2 = *reinterpret_cast<const f32x4 *>(&sm[(ow * 2 + 1) * TN * 32 + ocol]);
                        const float nbf = (float)nb, tot = rn + nbf;
                        const f32x4 delta = mb - rmean;
                        rmean += delta * (nbf / tot);
                        rm2 += d2 + delta * delta * (rn * nbf / tot);
                        rn = tot;
                    }
                }
                const int64_t tm = m0 / BM;
                *reinterpret_cast<f32x4 *>(p.stats + (tm * 2 + 0) * p.Nout + ncol) = rmean;
                *reinterpret_cast<f32x4 *>(p.stats + (tm * 2 + 1) * p.Nout + ncol) = rm2;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = rowdst[wm * TM * 32 + i * 32 + r];
        if (m < 0) continue;
        float *drow = dst + (int64_t)m * p.Nout;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int cbase = n0 + wn * TN * 32 + j * 32 + 4 * h;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = cbase + 8 * g;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (col + q < p.Nout) {
                        float val = acc[i][j][4 * g + q];
                        if (ACCUM) val = drow[col + q] + val;
                        drow[col + q] = val;
                    }
            }
        }
    }
}

template <int WGM, int WGN, int TM, int TN, int BKT, bool DGRAD>
hipError_t launch_igemm(IGemmP p, bool vec, int lin, bool accum, hipStream_t s, int *stats_tiles = nullptr)
{
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    const int tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.Nout + BN - 1) / BN;
    p.total_tiles = tiles_m * p.tiles_n;
    if (p.ksplit < 1) p.ksplit = 1;
    p.chunk = (p.total_tiles * p.ksplit + NXCD - 1) / NXCD;
    // volumes under a filter with depth: brick-shaped row tiles (every variant of the kernel addresses row by row)
    static const bool no_brick = getenv("POOCH_NO_BRICK") != nullptr;
    p.bd = 0;
    if (!no_brick && p.kd > 1 && BM % 64 == 0 && p.Dr % (BM / 64) == 0 && p.Hr % 8 == 0 && p.Wr % 8 == 0) p.bd = BM / 64;
    const dim3 grid(p.chunk * NXCD), block(64 * WGM * WGN);
    if (stats_tiles) {   // layout query of the statistics a STATS launch writes: row tiles, rows per tile
        stats_tiles[0] = tiles_m;
        stats_tiles[1] = BM;
        return hipSuccess;
    }
    if (p.stats) {
        if constexpr (!DGRAD) {
            if (!vec || lin == 0 || accum || p.dst_strided || p.Nout % 4 != 0) return hipErrorInvalidValue;
            if (lin == 2) igemm_kernel<WGM, WGN, TM, TN, BKT, true, 2, false, false, true><<<grid, block, 0, s>>>(p);
            else if (lin == 3) igemm_kernel<WGM, WGN, TM, TN, BKT, true, 3, false, false, true><<<grid, block, 0, s>>>(p);
            else igemm_kernel<WGM, WGN, TM, TN, BKT, true, 1, false, false, true><<<grid, block, 0, s>>>(p);
        } else {
            return hipErrorInvalidValue;
        }
    } else if (vec && lin == 2) {
        if constexpr (!DGRAD) {
            if (accum) return hipErrorInvalidValue;
            igemm_kernel<WGM, WGN, TM, TN, BKT, true, 2, false, false><<<grid, block, 0, s>>>(p);
        } else {
            return hipErrorInvalidValue;
        }
    } else if (vec && lin == 3) {
        if (accum) igemm_kernel<WGM, WGN, TM, TN, BKT, true, 3, DGRAD, true><<<grid, block, 0, s>>>(p);
        else igemm_kernel<WGM, WGN, TM, TN, BKT, true, 3, DGRAD, false><<<grid, block, 0, s>>>(p);
    } else if (vec && lin) {
        if (accum) igemm_kernel<WGM, WGN, TM, TN, BKT, true, 1, DGRAD, true><<<grid, block, 0, s>>>(p);
        else igemm_kernel<WGM, WGN, TM, TN, BKT, true, 1, DGRAD, false><<<grid, block, 0, s>>>(p);
    } else if (vec) {
        if (accum) igemm_kernel<WGM, WGN, TM, TN, BKT, true, 0, DGRAD, true><<<grid, block, 0, s>>>(p);
        else igemm_kernel<WGM, WGN, TM, TN, BKT, true, 0, DGRAD, false><<<grid, block, 0, s>>>(p);
    } else {
        if (accum) igemm_kernel<WGM, WGN, TM, TN, BKT, false, 0, DGRAD, true><<<grid, block, 0, s>>>(p);
        else igemm_kernel<WGM, WGN, TM, TN, BKT, false, 0, DGRAD, false><<<grid, block, 0, s>>>(p);
    }
    return hipGetLastError();
}

// the linear fast path of the vector kernel: whole slices per tap; the data gradient also needs unit strides
// 0: general; 1: whole slices per tap (the data gradient also needs unit strides); 2: several
// whole taps per slice (forward, plain write)
int igemm_linear_mode(int cs, bool dgrad, bool unit_stride, bool accum)
{
    static const bool off = getenv("POOCH_NO_LINEAR") != nullptr;
    if (off || cs % 4 != 0) return 0;
    if (cs % BK == 0) return (!dgrad || unit_stride) ? 1 : 0;
    if (BK % cs == 0 && !dgrad && !accum) return 2;
    return 0;
}

// Few tiles, long reduction (ResNet-50's last stages at batch 64, the deep levels of a 3-d CNN on one volume): 128 x 128
// tiles leave compute units idle and quarter-size tiles halve the flops per staged byte.  Such a GEMM keeps the 128 x 128
// tile and splits its reduction over ksplit workgroups per tile instead; each writes its partial result to a workspace
// and splitk_reduce_kernel adds the parts in a fixed order (deterministic, no atomics).  The convolution then leaves no
// batch-normalisation statistics (its tiles never see the finished values); these outputs are small, and the
// normalisation's own statistics pass over them costs microseconds.
constexpr size_t IGEMM_WS_CAP = (size_t)64 << 20;

struct SplitK {
    int ksplit, kslices;
};

SplitK igemm_splitk(int M, int Nout, int Kred, int lin, bool dst_strided)
{
    static const bool off = getenv("POOCH_NO_SPLITK") != nullptr;
    SplitK k{1, 0};
    if (off || lin != 1 || dst_strided || Nout <= 64 || Nout % 4 != 0) return k;
    const int64_t tiles = ((int64_t)(M + 127) / 128) * ((Nout + 127) / 128);
    const int nk = (Kred + BK - 1) / BK;
    // (a reduction of 2048: 81 TFLOP/s split against 85 with quarter-size tiles; 2304 and more: 89 - 106 against 60 - 90)
    // a handful of tiles (the FC layer: 640 x 1000 x 2048 is 40 tiles, one after the other 128 slices long): split whatever the
    // length, down to 8 slices per part
    const bool few = tiles < 64 && nk >= 32 && nk < 144;
    if (!few && (tiles >= 384 || nk < 144)) return k;
    int64_t want = (768 + tiles - 1) / tiles;                   // about three workgroups per compute unit
    if (want > (few ? 16 : 8)) want = few ? 16 : 8;
    const int min_slices = few ? 8 : 16;                        // at least 16 slices (256 reduction steps) per part
    if (want > nk / min_slices) want = nk / min_slices;
    const int64_t by_ws = (int64_t)(IGEMM_WS_CAP / ((size_t)M * Nout * sizeof(float)));
    if (want > by_ws) want = by_ws;
    if (want < 2) return k;
    k.kslices = (int)((nk + want - 1) / want);
    k.ksplit = (nk + k.kslices - 1) / k.kslices;
    if (k.ksplit < 2) k = SplitK{1, 0};
    return k;
}

// dst[i] (+)= ((part[0][i] + part[1][i]) + part[2][i]) + ...: one float4 per thread
template <bool ACCUM>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, float *__restrict__ dst, int64_t n4, int ksplit)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    const f32x4 *pp = reinterpret_cast<const f32x4 *>(part);
    f32x4 v = __builtin_nontemporal_load(pp + i);
    for (int k = 1; k < ksplit; ++k) v += __builtin_nontemporal_load(pp + (int64_t)k * n4 + i);
    f32x4 *dp = reinterpret_cast<f32x4 *>(dst) + i;
    if (ACCUM) v = *dp + v;
    __builtin_nontemporal_store(v, dp);
}

// ---- 3 x 3 x 3, unit stride, padding 1, 32 -> 32 channels: the input brick stays in LDS ---------------------------------
// The first level of a 3-d CNN on a 192^3 volume: the reduction is only 864 long, so igemm_kernel stages 27 slices
// per tile through LDS with a barrier after each and runs at about 105 TFLOP/s.  Here a workgroup of four waves owns
// a brick of 2 x 8 x 8 output positions (128 GEMM rows, one 32 x 32 block per wave).  It loads the 4 x 10 x 10 input
// positions the brick's 27 taps touch into LDS ONCE (57.6 KB with rows padded to 36 floats: two workgroups per CU),
// and the tap loop then reads its A operand straight from that copy -- no staging, no barrier, no address arithmetic
// beyond a constant per tap.  The B operand (one tap's 32 x 32 filter slice, 4 KB) comes from global memory through
// the caches, a tap ahead, like A.  Lane (r, h) feeds reduction steps (c = t, c = 16 + t) for t = 0..15, so both of
// its operands are 64 contiguous bytes.
// The data gradient is the same convolution over dy with the taps mirrored (position tap t' uses filter tap 26 - t')
// and the transposed filter copy, which has the same [out][tap][in] layout.
// Measured on 1 x 192^3 x 32 (stand-alone, warm clocks): 124 TFLOP/s against 105 for igemm_kernel; with LDS filled
// from registers instead of global memory and no stores the same loop runs at 130, so little is left in this design.
// (Two variants that were not kept: a persistent workgroup that prefetches the next brick into registers during the
// tap loop -- 109 TFLOP/s, the in-order counter of outstanding loads makes the filter loads wait for the brick's --
// and a swizzled, unpadded brick that admits three workgroups per CU -- 118.  Wider layers through the same brick space --
// source channels in groups of 32, two or four blocks of 32 output channels per wave -- ran at 100 TFLOP/s (64 output
// channels) and 69 (128) against igemm_kernel's 114 and 108 at 96^3 and 48^3: every wave then loads 8 or 16 KB of filter
// per tap from the L2, where igemm_kernel stages a slice once per workgroup.)
constexpr int C3_BD = 2, C3_BH = 8, C3_BW = 8, C3_C = 32;
constexpr int C3_HD = C3_BD + 2, C3_HH = C3_BH + 2, C3_HW = C3_BW + 2, C3_NPIX = C3_HD * C3_HH * C3_HW;
constexpr int C3_LP = 36;   // floats per pixel in LDS: 16-byte aligned, and eight consecutive pixels start in different banks

// The results of a 2 x 8 x 8 brick (four waves, one 32 x 32 accumulator block each; wave w holds rows 32 w .. 32 w + 31 of the
// brick, w fastest) leave through `lds` (4 x 32 x C3_LP floats that no wave reads any more), so that a store covers whole
// 128-byte rows.  Accumulator element v of lane (r, h) is output channel 8 * (v / 4) + 4 * h + v % 4 of row r.
// STATS: mean and sum of squared deviations (M2) of the brick's 128 rows per channel, in igemm_kernel's format: per wave over
// its 32 rows (mean first, then M2 about it), the four waves merged in order by the pairwise update of Chan et al.
template <bool ACCUM, bool STATS>
__device__ __forceinline__ void c3_brick_out(const f32x16 &acc, float *lds, const IGemmP &p, int wave, int lane, int n, int d0, int h0, int w0)
{
    const int r = lane % 32, h = lane / 32;
    const int D = p.Dr, H = p.Hr, W = p.Wr;
    float *cw = lds + wave * 32 * C3_LP;
    const int orow = lane / 8, ocol = 4 * (lane % 8);
    // accumulating: the old values are requested together before the block goes through LDS (a load placed between the
    // stores waits for the store before it, one memory round trip per row group)
    f32x4 oldv[ACCUM ? 4 : 1];
    if constexpr (ACCUM) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = wave * 32 + q * 8 + orow;
            const int64_t m = (((int64_t)n * D + d0 + row / 64) * H + h0 + (row / 8) % 8) * W + w0 + row % 8;
            oldv[q] = __builtin_nontemporal_load((gvec4_ptr)(p.dst + m * C3_C + ocol));
        }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 val = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
        *reinterpret_cast<f32x4 *>(&cw[r * C3_LP + 8 * g + 4 * h]) = val;
    }
    __syncthreads();
    f32x4 vq[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = wave * 32 + q * 8 + orow;
        const int64_t m = (((int64_t)n * D + d0 + row / 64) * H + h0 + (row / 8) % 8) * W + w0 + row % 8;
        f32x4 val = *reinterpret_cast<const f32x4 *>(&cw[(q * 8 + orow) * C3_LP + ocol]);
        vq[q] = val;
        f32x4 *dp = reinterpret_cast<f32x4 *>(p.dst + m * C3_C + ocol);
        if constexpr (ACCUM) val = oldv[q] + val;
        __builtin_nontemporal_store(val, dp);
    }
    if constexpr (STATS) {
        f32x4 sum = (vq[0] + vq[1]) + (vq[2] + vq[3]);
#pragma unroll
        for (int mask = 8; mask < 64; mask <<= 1) {
            sum.x += __shfl_xor(sum.x, mask, 64); sum.y += __shfl_xor(sum.y, mask, 64);
            sum.z += __shfl_xor(sum.z, mask, 64); sum.w += __shfl_xor(sum.w, mask, 64);
        }
        f32x4 rmean = sum / 32.f;
        f32x4 rm2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 d = vq[q] - rmean;
            rm2 += d * d;
        }
#pragma unroll
        for (int mask = 8; mask < 64; mask <<= 1) {
            rm2.x += __shfl_xor(rm2.x, mask, 64); rm2.y += __shfl_xor(rm2.y, mask, 64);
            rm2.z += __shfl_xor(rm2.z, mask, 64); rm2.w += __shfl_xor(rm2.w, mask, 64);
        }
        __syncthreads();                                  // the staging rows have been read
        float *sm = lds;                                  // [wave][mean, M2][32]
        if (orow == 0) {
            *reinterpret_cast<f32x4 *>(&sm[(wave * 2 + 0) * 32 + ocol]) = rmean;
            *reinterpret_cast<f32x4 *>(&sm[(wave * 2 + 1) * 32 + ocol]) = rm2;
        }
        __syncthreads();
        if (wave == 0 && orow == 0) {
            float rn = 32.f;
#pragma unroll
            for (int w2 = 1; w2 < 4; ++w2) {
                const f32x4 mb = *reinterpret_cast<const f32x4 *>(&sm[(w2 * 2 + 0) * 32 + ocol]);
                const f32x4 d2 = *reinterpret_cast<const f32x4 *>(&sm[(w2 * 2 + 1) * 32 + ocol]);
                const float tot = rn + 32.f;
                const f32x4 delta = mb - rmean;
                rmean += delta * (32.f / tot);
                rm2 += d2 + delta * delta * (rn * 32.f / tot);
                rn = tot;
            }
            const int64_t tm = blockIdx.x;
            *reinterpret_cast<f32x4 *>(p.stats + (tm * 2 + 0) * C3_C + ocol) = rmean;
            *reinterpret_cast<f32x4 *>(p.stats + (tm * 2 + 1) * C3_C + ocol) = rm2;
        }
    }
}

template <bool DGRAD, bool ACCUM, bool STATS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv3_halo_kernel(IGemmP p)
{
    __shared__ __attribute__((aligned(16))) float brick[C3_NPIX * C3_LP];
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int D = p.Dr, H = p.Hr, W = p.Wr;
    const int nbw = W / C3_BW, nbh = H / C3_BH, nbd = D / C3_BD;
    int t = blockIdx.x;
    const int w0 = (t % nbw) * C3_BW; t /= nbw;
    const int h0 = (t % nbh) * C3_BH; t /= nbh;
    const int d0 = (t % nbd) * C3_BD;
    const int n = t / nbd;
    const float *x = p.src + (int64_t)n * D * H * W * C3_C;
    {
        // a halo line (pd, ph) is 10 pixels = 1280 contiguous bytes = 80 lanes x 16 bytes; wave w takes lines w, w + 4, ...
        // (line numbers, validity and addresses are wave-uniform: scalar arithmetic)
        constexpr int NL = C3_HD * C3_HH / 4;
        f32x4 v0[NL], v1[NL];
        const int pw0 = lane / 8, q4 = 4 * (lane % 8);
        const bool in0 = !(w0 == 0 && pw0 == 0);                          // pixel w0 - 1 + pw0, pw0 = 0..7
        const bool in1 = lane < 16 && !(w0 + C3_BW == W && pw0 == 1);     // pixels w0 + 7 and w0 + 8
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            const int line = wave + 4 * k, pd = line / C3_HH, ph = line % C3_HH;
            const int id = d0 + pd - 1, ih = h0 + ph - 1;
            const bool lok = (unsigned)id < (unsigned)D && (unsigned)ih < (unsigned)H;
            const float *src = x + ((((int64_t)(lok ? id : 0) * H + (lok ? ih : 0)) * W + w0) * C3_C - C3_C);
            v0[k] = (lok && in0) ? ldg4(src + 4 * lane) : z;
            v1[k] = (lok && in1) ? ldg4(src + 4 * lane + 256) : z;
        }
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            const int line = wave + 4 * k;
            float *dst = brick + (line * C3_HW + pw0) * C3_LP + q4;
            *reinterpret_cast<f32x4 *>(dst) = v0[k];
            if (lane < 16) *reinterpret_cast<f32x4 *>(dst + 8 * C3_LP) = v1[k];
        }
    }
    __syncthreads();
    const int R = wave * 32 + r;                                          // this lane's GEMM row within the brick
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float *abase = brick + (((R / 64) * C3_HH + (R / 8) % 8) * C3_HW + R % 8) * C3_LP + h * 16;
    const float *bbase = p.wgt + (r * 27 * C3_C + h * 16);
    f32x4 a0[4], b0[4], a1[4], b1[4];
    auto load = [&](f32x4 (&a)[4], f32x4 (&b)[4], int tap) {
        const int ta = tap / 9, tb = (tap / 3) % 3, te = tap % 3;
        const float *ap = abase + ((ta * C3_HH + tb) * C3_HW + te) * C3_LP;
        const float *bp = bbase + (DGRAD ? 26 - tap : tap) * C3_C;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = *reinterpret_cast<const f32x4 *>(ap + 4 * i);
            b[i] = ldg4(bp + 4 * i);
        }
    };
    auto mul = [&](const f32x4 (&a)[4], const f32x4 (&b)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(b[i][j], a[i][j], acc, 0, 0, 0);
    };
    // loads of tap t + 1 are issued before the MFMAs of tap t; the fences keep the compiler from sinking them to their
    // first use (which it does to save registers, and which leaves every tap waiting for its own loads)
    load(a0, b0, 0);
#pragma unroll 1
    for (int tap = 0; tap < 26; tap += 2) {
        load(a1, b1, tap + 1);
        __builtin_amdgcn_sched_barrier(0);
        mul(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        load(a0, b0, tap + 2);
        __builtin_amdgcn_sched_barrier(0);
        mul(a1, b1);
        __builtin_amdgcn_sched_barrier(0);
    }
    mul(a0, b0);

    __syncthreads();                                      // every wave is done with the brick: its space becomes the staging area
    c3_brick_out<ACCUM, STATS>(acc, brick, p, wave, lane, n, d0, h0, w0);
}

// ---- the same filter shape on a network input with ONE live channel (a volume of intensities), 32 output channels ----------
// The reduction is 27 values long.  As a GEMM over the stored four channels (three of them zero) it is 108 long and runs
// igemm_kernel at 19 TFLOP/s: 0.63 ms for 0.9 GB of output on 192^3, a third of the HBM rate.  Here the brick's halo is 400
// floats in LDS, a lane gathers its pixel's 27 neighbours from there (reduction steps (2 t, 2 t + 1), the 28th weight is
// zero), the 27 x 32 filter sits in 14 registers per lane, and a brick costs 14 MFMAs per wave: what remains is writing the
// result (and its statistics), which is the bound.
template <bool STATS>
__global__ __launch_bounds__(256) void conv3_c1_kernel(IGemmP p)
{
    __shared__ __attribute__((aligned(16))) float lds[4 * 32 * C3_LP];      // the halo (400 floats), later the staging rows
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int D = p.Dr, H = p.Hr, W = p.Wr, CS = p.Cs;
    const int nbw = W / C3_BW, nbh = H / C3_BH, nbd = D / C3_BD;
    int t = blockIdx.x;
    const int w0 = (t % nbw) * C3_BW; t /= nbw;
    const int h0 = (t % nbh) * C3_BH; t /= nbh;
    const int d0 = (t % nbd) * C3_BD;
    const int n = t / nbd;
    const float *x = p.src + (int64_t)n * D * H * W * CS;
    for (int u = tid; u < C3_NPIX; u += 256) {
        const int id = d0 + u / (C3_HH * C3_HW) - 1, ih = h0 + (u / C3_HW) % C3_HH - 1, iw = w0 + u % C3_HW - 1;
        const bool ok = (unsigned)id < (unsigned)D && (unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W;
        lds[u] = ok ? ldg1(x + (((int64_t)id * H + ih) * W + iw) * CS) : 0.f;
    }
    float bw[14];
#pragma unroll
    for (int k = 0; k < 14; ++k) {
        const int tap = 2 * k + h;
        bw[k] = tap < 27 ? ldg1(p.wgt + ((int64_t)r * 27 + tap) * CS) : 0.f;
    }
    __syncthreads();
    const int R = wave * 32 + r;
    const int pbase = ((R / 64) * C3_HH + (R / 8) % 8) * C3_HW + R % 8;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    float af[14];
#pragma unroll
    for (int k = 0; k < 14; ++k) {
        // (the 28th step of the h = 1 lanes reads the 27th neighbour again; its weight is zero)
        const int t0 = 2 * k, t1 = 2 * k + 1 < 27 ? 2 * k + 1 : 26;
        const int o0 = ((t0 / 9) * C3_HH + (t0 / 3) % 3) * C3_HW + t0 % 3, o1 = ((t1 / 9) * C3_HH + (t1 / 3) % 3) * C3_HW + t1 % 3;
        af[k] = lds[pbase + (h ? o1 : o0)];
    }
#pragma unroll
    for (int k = 0; k < 14; ++k) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bw[k], af[k], acc, 0, 0, 0);
    __syncthreads();                                      // the halo has been read: its space becomes the staging area
    c3_brick_out<false, STATS>(acc, lds, p, wave, lane, n, d0, h0, w0);
}

// the geometry the brick kernels are written for: 3 x 3 x 3, unit stride, padding 1, output extents = input extents in whole
// 2 x 8 x 8 bricks, 32 output channels (small volumes too: 128-row bricks give a short launch more workgroups than
// igemm_kernel's 256-row tiles)
bool c3_brick_geom(const IGemmP &p)
{
    if (p.dst_strided || p.Nout != C3_C) return false;
    if (p.kd != 3 || p.kh != 3 || p.kw != 3 || p.sd != 1 || p.sh != 1 || p.sw != 1 || p.pd != 1 || p.ph != 1 || p.pw != 1) return false;
    if (p.Ds != p.Dr || p.Hs != p.Hr || p.Ws != p.Wr) return false;
    if (p.Dr % C3_BD != 0 || p.Hr % C3_BH != 0 || p.Wr % C3_BW != 0) return false;
    return p.M >= C3_BD * C3_BH * C3_BW;
}

bool conv3_halo_ok(const IGemmP &p, bool vec)
{
    static const bool off = getenv("POOCH_NO_CONV3_HALO") != nullptr;
    return !off && vec && c3_brick_geom(p) && p.Cs == C3_C && p.Kred == 27 * C3_C;
}

// forward over a source of which only the first channel is live
bool conv3_c1_ok(const IGemmP &p)
{
    static const bool off = getenv("POOCH_NO_CONV3_C1") != nullptr;
    return !off && p.live == 1 && c3_brick_geom(p) && p.Kred == 27 * p.Cs;
}

template <bool DGRAD>
hipError_t launch_conv3_halo(const IGemmP &p, bool accum, hipStream_t s, int *stats_tiles)
{
    const int bricks = p.M / (C3_BD * C3_BH * C3_BW);
    if (stats_tiles) {
        stats_tiles[0] = bricks;
        stats_tiles[1] = C3_BD * C3_BH * C3_BW;
        return hipSuccess;
    }
    const dim3 grid(bricks), block(256);
    if constexpr (DGRAD) {
        if (p.stats) return hipErrorInvalidValue;
        if (accum) conv3_halo_kernel<true, true, false><<<grid, block, 0, s>>>(p);
        else conv3_halo_kernel<true, false, false><<<grid, block, 0, s>>>(p);
    } else {
        if (accum) return hipErrorInvalidValue;
        if (p.stats) conv3_halo_kernel<false, false, true><<<grid, block, 0, s>>>(p);
        else conv3_halo_kernel<false, false, false><<<grid, block, 0, s>>>(p);
    }
    return hipGetLastError();
}

// ---- the ResNet stem: 7 x 7, stride 2, padding 3, three live input channels (stored as four), 64 output channels ----------
// As a GEMM over the stored channels the reduction is 196 long (13 slices of 16) for 147 live values, staged per slice:
// igemm_kernel runs it at 73 TFLOP/s of live flops (2.07 ms at batch 640).  Here a workgroup takes a tile of 8 x 16 output
// positions, brings the 21 x 37 input pixels under it into LDS once -- one plane per channel and column parity, so that the
// 16 positions of a tile row read consecutive floats for any tap (x = 2 ox + tx: parity tx % 2, index ox + tx / 2) -- and a
// lane gathers its position's 147 values from there: 74 reduction steps, lanes 0 - 31 the values 0 .. 73, lanes 32 - 63 the
// values 74 .. 146 and a zero.  Wave w holds output channels 32 (w / 2) .. + 31 for the tile's rows 64 (w % 2) .. + 63 (two
// accumulator blocks), so its share of the filter is 74 registers per lane, loaded once: workgroups are persistent.
constexpr int S7_TH = 8, S7_TW = 16, S7_PH = 2 * S7_TH + 5, S7_PW = 2 * S7_TW + 5, S7_RS = 24;   // tile, patch, plane row stride
constexpr int S7_PATCH = 3 * 2 * S7_PH * S7_RS;                                                   // floats

// offset in the patch planes of reduction value k = 3 * tap + c (tap = 7 ty + tx), relative to a position's base
__host__ __device__ constexpr int s7_off(int k)
{
    return k >= 147 ? 0 : (((k % 3) * 2 + ((k / 3) % 7) % 2) * S7_PH + (k / 3) / 7) * S7_RS + ((k / 3) % 7) / 2;
}

template <bool STATS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void stem7_fwd_kernel(IGemmP p, int tiles, int per_wg)
{
    __shared__ __attribute__((aligned(16))) float patch[S7_PATCH];
    __shared__ __attribute__((aligned(16))) float stage[4 * 32 * C3_LP];
    __shared__ __attribute__((aligned(16))) float sm[4 * 2 * 32];
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int nb = wave / 2, half = wave % 2;
    const int Ho = p.Hr, Wo = p.Wr, H = p.Hs, W = p.Ws, CS = p.Cs, NO = p.Nout;
    const int tw = Wo / S7_TW, th = Ho / S7_TH;
    float bw[74];
#pragma unroll
    for (int t = 0; t < 74; ++t) {
        const int k = 74 * h + t;
        bw[t] = k < 147 ? ldg1(p.wgt + ((int64_t)(32 * nb + r) * 49 + k / 3) * CS + k % 3) : 0.f;
    }
    // rows of this lane: R = 64 half + 32 b + r (b = 0, 1): tile row R / 16, column R % 16; block 1 is two tile rows further down
    const int R0 = 64 * half + r;
    const float *abase = patch + (2 * (R0 / S7_TW)) * S7_RS + R0 % S7_TW;
    const int t_end = min((int)(blockIdx.x + 1) * per_wg, tiles);
    // the pixels of a tile's patch travel global -> registers while the tile before it is multiplied (four per thread), and
    // go to the planes between two barriers
    constexpr int NPF = (S7_PH * S7_PW + 255) / 256;
    f32x4 pf[NPF];
    auto fetch = [&](int tile) {
        int t = tile;
        const int ox0 = (t % tw) * S7_TW; t /= tw;
        const int oy0 = (t % th) * S7_TH;
        const float *x = p.src + (int64_t)(t / th) * H * W * CS;
#pragma unroll
        for (int j = 0; j < NPF; ++j) {
            const int u = tid + 256 * j, py = u / S7_PW, px = u % S7_PW;
            const int iy = 2 * oy0 - 3 + py, ix = 2 * ox0 - 3 + px;
            const bool ok = u < S7_PH * S7_PW && (unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            pf[j] = ok ? ldg4(x + ((int64_t)iy * W + ix) * CS) : z;
        }
    };
    if ((int)blockIdx.x * per_wg < t_end) fetch(blockIdx.x * per_wg);
    for (int tile = blockIdx.x * per_wg; tile < t_end; ++tile) {
        int t = tile;
        const int ox0 = (t % tw) * S7_TW; t /= tw;
        const int oy0 = (t % th) * S7_TH;
        const int n = t / th;
        __syncthreads();                                  // the previous tile's patch has been read
#pragma unroll
        for (int j = 0; j < NPF; ++j) {
            const int u = tid + 256 * j, py = u / S7_PW, px = u % S7_PW;
            if (u < S7_PH * S7_PW) {
                float *d = patch + ((px & 1) * S7_PH + py) * S7_RS + (px >> 1);
                d[0] = pf[j].x;
                d[2 * S7_PH * S7_RS] = pf[j].y;
                d[4 * S7_PH * S7_RS] = pf[j].z;
            }
        }
        __syncthreads();
        fetch(min(tile + 1, t_end - 1));                  // (the last tile again: no branch around the loads)
        f32x16 acc[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
#pragma unroll
        for (int t2 = 0; t2 < 74; ++t2) {
            const int off = h ? s7_off(74 + t2) : s7_off(t2);
            const float a0 = abase[off], a1 = abase[off + 4 * S7_RS];
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bw[t2], a0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bw[t2], a1, acc[1], 0, 0, 0);
        }
        // element v of lane (r, h): output channel 32 nb + 8 (v / 4) + 4 h + v % 4 of row r of the block.  Through this wave's
        // staging rows (LDS serves a wave's instructions in order), so that a store covers 128-byte pieces of output rows.
        float *cw = stage + wave * 32 * C3_LP;
        const int orow = lane / 8, ocol = 4 * (lane % 8);
        float rn = 0.f;
        f32x4 rmean = {0.f, 0.f, 0.f, 0.f}, rm2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 val = {acc[b][4 * g], acc[b][4 * g + 1], acc[b][4 * g + 2], acc[b][4 * g + 3]};
                *reinterpret_cast<f32x4 *>(&cw[r * C3_LP + 8 * g + 4 * h]) = val;
            }
            __builtin_amdgcn_wave_barrier();
            f32x4 vq[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int R = 64 * half + 32 * b + 8 * q + orow;
                const int64_t m = ((int64_t)n * Ho + oy0 + R / S7_TW) * Wo + ox0 + R % S7_TW;
                vq[q] = *reinterpret_cast<const f32x4 *>(&cw[(8 * q + orow) * C3_LP + ocol]);
                __builtin_nontemporal_store(vq[q], reinterpret_cast<f32x4 *>(p.dst + m * NO + 32 * nb + ocol));
            }
            __builtin_amdgcn_wave_barrier();
            if constexpr (STATS) {
                f32x4 sum = (vq[0] + vq[1]) + (vq[2] + vq[3]);
#pragma unroll
                for (int mask = 8; mask < 64; mask <<= 1) {
                    sum.x += __shfl_xor(sum.x, mask, 64); sum.y += __shfl_xor(sum.y, mask, 64);
                    sum.z += __shfl_xor(sum.z, mask, 64); sum.w += __shfl_xor(sum.w, mask, 64);
                }
                const f32x4 mb = sum / 32.f;
                f32x4 d2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 d = vq[q] - mb;
                    d2 += d * d;
                }
#pragma unroll
                for (int mask = 8; mask < 64; mask <<= 1) {
                    d2.x += __shfl_xor(d2.x, mask, 64); d2.y += __shfl_xor(d2.y, mask, 64);
                    d2.z += __shfl_xor(d2.z, mask, 64); d2.w += __shfl_xor(d2.w, mask, 64);
                }
                const float tot = rn + 32.f;
                const f32x4 delta = mb - rmean;
                rmean += delta * (32.f / tot);
                rm2 += d2 + delta * delta * (rn * 32.f / tot);
                rn = tot;
            }
        }
        if constexpr (STATS) {
            // mean and M2 of the tile's 128 rows per channel (igemm_kernel's format): the two waves of a column block, in order
            if (orow == 0) {
                *reinterpret_cast<f32x4 *>(&sm[(wave * 2 + 0) * 32 + ocol]) = rmean;
                *reinterpret_cast<f32x4 *>(&sm[(wave * 2 + 1) * 32 + ocol]) = rm2;
            }
            __syncthreads();
            if (half == 0 && orow == 0) {
                const f32x4 mb = *reinterpret_cast<const f32x4 *>(&sm[((wave + 1) * 2 + 0) * 32 + ocol]);
                const f32x4 d2 = *reinterpret_cast<const f32x4 *>(&sm[((wave + 1) * 2 + 1) * 32 + ocol]);
                const f32x4 delta = mb - rmean;
                rmean += delta * 0.5f;
                rm2 += d2 + delta * delta * 32.f;             // 64 * 64 / 128
                *reinterpret_cast<f32x4 *>(p.stats + ((int64_t)tile * 2 + 0) * NO + 32 * nb + ocol) = rmean;
                *reinterpret_cast<f32x4 *>(p.stats + ((int64_t)tile * 2 + 1) * NO + 32 * nb + ocol) = rm2;
            }
        }
    }
}

bool stem7_ok(const IGemmP &p)
{
    static const bool off = getenv("POOCH_NO_STEM7") != nullptr;
    if (off || p.dst_strided || p.live != 3 || p.Cs != 4 || p.Nout != 64 || p.Kred != 49 * 4) return false;
    if (p.kd != 1 || p.kh != 7 || p.kw != 7 || p.sd != 1 || p.sh != 2 || p.sw != 2 || p.pd != 0 || p.ph != 3 || p.pw != 3) return false;
    if (p.Dr != 1 || p.Ds != 1 || p.Hs != 2 * p.Hr || p.Ws != 2 * p.Wr) return false;
    if (p.Hr % S7_TH != 0 || p.Wr % S7_TW != 0) return false;
    return (uintptr_t)p.src % 16 == 0;
}

hipError_t launch_stem7(const IGemmP &p, hipStream_t s, int *stats_tiles)
{
    const int tiles = p.M / (S7_TH * S7_TW);
    if (stats_tiles) {
        stats_tiles[0] = tiles;
        stats_tiles[1] = S7_TH * S7_TW;
        return hipSuccess;
    }
    const int nwg = tiles < 2 * NCU ? tiles : 2 * NCU;          // persistent (two workgroups fit a compute unit): the filter is loaded once each
    const int per_wg = (tiles + nwg - 1) / nwg;
    const dim3 grid((tiles + per_wg - 1) / per_wg), block(256);
    if (p.stats) stem7_fwd_kernel<true><<<grid, block, 0, s>>>(p, tiles, per_wg);
    else stem7_fwd_kernel<false><<<grid, block, 0, s>>>(p, tiles, per_wg);
    return hipGetLastError();
}

hipError_t launch_conv3_c1(const IGemmP &p, hipStream_t s, int *stats_tiles)
{
    const int bricks = p.M / (C3_BD * C3_BH * C3_BW);
    if (stats_tiles) {
        stats_tiles[0] = bricks;
        stats_tiles[1] = C3_BD * C3_BH * C3_BW;
        return hipSuccess;
    }
    if (p.stats) conv3_c1_kernel<true><<<dim3(bricks), dim3(256), 0, s>>>(p);
    else conv3_c1_kernel<false><<<dim3(bricks), dim3(256), 0, s>>>(p);
    return hipGetLastError();
}

template <bool DGRAD>
hipError_t dispatch_igemm(const IGemmP &p0, bool accum, hipStream_t s, int *stats_tiles = nullptr, float *workspace = nullptr)
{
    IGemmP p = p0;
    p.ksplit = 1;
    p.kslices = 0;
    const bool vec = (p.Cs % 4 == 0) && ((uintptr_t)p.src % 16 == 0) && ((uintptr_t)p.wgt % 16 == 0);
    int lin = vec ? igemm_linear_mode(p.Cs, DGRAD, p.sd == 1 && p.sh == 1 && p.sw == 1, accum) : 0;
    const SplitK sk = igemm_splitk(p.M, p.Nout, p.Kred, lin, p.dst_strided != 0);
    static const bool no_gemm = getenv("POOCH_NO_GEMM_PATH") != nullptr;
    if (lin == 1 && !no_gemm && p.kd * p.kh * p.kw == 1 && p.pd == 0 && p.ph == 0 && p.pw == 0) lin = 3;   // one tap, no padding
    if (sk.ksplit > 1) {
        if (stats_tiles || p.stats) return hipErrorInvalidValue;      // no statistics from a split reduction
        if (!workspace || (uintptr_t)workspace % 16 != 0 || (uintptr_t)p.dst % 16 != 0) return hipErrorInvalidValue;
        float *const final_dst = p.dst;
        p.dst = workspace;
        p.ksplit = sk.ksplit;
        p.kslices = sk.kslices;
        const hipError_t e = launch_igemm<2, 2, 2, 2, BK, DGRAD>(p, vec, lin, false, s, nullptr);
        if (e != hipSuccess) return e;
        const int64_t n4 = (int64_t)p.M * p.Nout / 4;
        const dim3 grid((unsigned)((n4 + 255) / 256));
        if (accum) splitk_reduce_kernel<true><<<grid, dim3(256), 0, s>>>(workspace, final_dst, n4, sk.ksplit);
        else splitk_reduce_kernel<false><<<grid, dim3(256), 0, s>>>(workspace, final_dst, n4, sk.ksplit);
        return hipGetLastError();
    }
    // too few 128x128 tiles to fill 256 compute units three workgroups deep: quarter-size tiles
    if (p.Nout > 64 && ((int64_t)(p.M + 127) / 128) * ((p.Nout + 127) / 128) < 640) return launch_igemm<2, 2, 1, 1, BK, DGRAD>(p, vec, lin, accum, s, stats_tiles);
    // 32 output channels: a wave holds two accumulator blocks, so a 16-wide slice is only 16 MFMAs between two barriers; 32-wide
    // slices where a tap spans whole ones (3 x 3 x 3, 32 -> 32 at 192^3: forward 104 -> 108 TFLOP/s, data gradient 98 -> 108;
    // the wider tiles lose 3 % under 3 x 3 filters and gain 1 % at most under 1 x 1)
    if (p.Nout <= 32) {
        if (conv3_halo_ok(p, vec) && !(accum && !DGRAD)) return launch_conv3_halo<DGRAD>(p, accum, s, stats_tiles);
        if (!DGRAD && !accum && conv3_c1_ok(p)) return launch_conv3_c1(p, s, stats_tiles);
        static const bool narrow = getenv("POOCH_NO_WIDE_SLICE") != nullptr;
        if (!narrow && lin == 1 && p.Cs % 32 == 0) return launch_igemm<4, 1, 2, 1, 32, DGRAD>(p, vec, lin, accum, s, stats_tiles);
        return launch_igemm<4, 1, 2, 1, BK, DGRAD>(p, vec, lin, accum, s, stats_tiles);
    }
    if (!DGRAD && !accum && stem7_ok(p)) return launch_stem7(p, s, stats_tiles);
    if (p.Nout <= 64) return launch_igemm<4, 1, 2, 2, BK, DGRAD>(p, vec, lin, accum, s, stats_tiles);
    return launch_igemm<2, 2, 2, 2, BK, DGRAD>(p, vec, lin, accum, s, stats_tiles);
}

// one float4 per thread, no loop: short-lived blocks stream closest to the HBM peak
__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, int64_t n)
{
    const int64_t n4 = n / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(f32x4{0.f, 0.f, 0.f, 0.f}, reinterpret_cast<f32x4 *>(p) + i);
    if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) p[n4 * 4 + threadIdx.x] = 0.f;
}

hipError_t fill_zero(float *p, int64_t n, hipStream_t s)
{
    if ((uintptr_t)p % 16 != 0 || n < 0 || n >= ((int64_t)1 << 40)) return hipErrorInvalidValue;
    int64_t blocks = (n / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    fill_zero_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(p, n);
    return hipGetLastError();
}

bool geom_ok(const ConvGeom &g)
{
    if (g.N <= 0 || g.C <= 0 || g.K <= 0 || g.D <= 0 || g.H <= 0 || g.W <= 0) return false;
    if (g.kd <= 0 || g.kh <= 0 || g.kw <= 0 || g.sd <= 0 || g.sh <= 0 || g.sw <= 0) return false;
    if (g.pd < 0 || g.ph < 0 || g.pw < 0) return false;
    if (g.Do != (g.D + 2 * g.pd - g.kd) / g.sd + 1 || g.Ho != (g.H + 2 * g.ph - g.kh) / g.sh + 1 ||
        g.Wo != (g.W + 2 * g.pw - g.kw) / g.sw + 1)
        return false;
    if (g.Do <= 0 || g.Ho <= 0 || g.Wo <= 0) return false;
    // row indices and reduction lengths are 32-bit inside the kernels
    const int64_t lim = (int64_t)1 << 31;
    if (g.rows_out() >= lim - 4096 || g.rows_in() >= lim - 4096) return false;
    if (g.taps() * g.C >= lim || g.taps() * g.K >= lim) return false;
    return true;
}

// ------------------------------------------------------------------ filter gradient

struct WGradP {
    const float *dy;  // [M][K]
    const float *x;   // channels-last input
    float *out;       // nsplit == 1: dw [K][Kred]; else partials [nsplit][K][Kred]
    int M, K, Kred, C;
    int Do, Ho, Wo, D, H, W;
    int kd, kh, kw, sd, sh, sw, pd, ph, pw;
    int tiles_n, chunk_rows, nsplit;
    int tiles, total, chunk;  // tiles per split, workgroups that have work, workgroups per XCD
};

template <int WGM, int WGN, int TM, int TN, bool VECA, bool VECB>
__global__ __launch_bounds__(64 * WGM * WGN) void wgrad_kernel(WGradP p)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;  // BM over output channels, BN over taps*C
    constexpr int LDA = (BM + 63) / 64 * 64 + 32, LDB = (BN + 63) / 64 * 64 + 32;
    constexpr int A_V = 4 * BM / NT, B_V = 4 * BN / NT, A_S = 16 * BM / NT, B_S = 16 * BN / NT;
    static_assert(4 * BM % NT == 0 && 4 * BN % NT == 0, "tile/threads mismatch");
    // the vector paths give every thread one fixed column of each operand for all its passes
    static_assert(NT % (BM / 4) == 0 && NT % (BN / 4) == 0, "a thread's column must not depend on the pass");

    __shared__ __attribute__((aligned(16))) float As[BK * LDA];
    __shared__ __attribute__((aligned(16))) float Bs[BK * LDB];
    // fast path (both operands vectorised): where the rows of the next SEG reduction steps start
    // in x -- element offset of the window's first tap and that tap's coordinates -- computed once
    // per segment so that the main loop has no divisions
    constexpr bool TAB = VECA && VECB;
    constexpr int SEG = 512;
    __shared__ int4 rowc[TAB ? SEG : 1];
    __shared__ int64_t rowb[TAB ? SEG : 1];

    const int tid = threadIdx.x;
    // all tiles of one split run next to each other on one XCD: they stream the same rows of dy and
    // (shifted by a tap) of x, which its L2 then fetches once instead of once per tile
    const int logical = remap_tile(blockIdx.x, p.chunk);
    if (logical >= p.total) return;
    const int tile = logical % p.tiles, split = logical / p.tiles;
    const int k0 = (tile / p.tiles_n) * BM;  // first output channel of the tile
    const int j0 = (tile % p.tiles_n) * BN;  // first (tap, c) column of the tile
    const int mbeg = split * p.chunk_rows;
    const int mend = min(p.M, mbeg + p.chunk_rows);

    float4 av[VECA ? A_V : 1], bv[VECB ? B_V : 1];
    float as[VECA ? 1 : A_S], bs[VECB ? 1 : B_S];
    f32x4 tav[A_V], tbv[B_V];   // prefetch registers of the fast path (native vectors: they must stay registers)

    // column of x-patches this thread gathers (fixed for the whole kernel in the VECB path)
    int vb_a = 0, vb_b = 0, vb_e = 0, vb_c = 0;
    bool vb_ok = false;
    if (VECB) {
        const int col = j0 + 4 * (tid % (BN / 4));
        vb_ok = col < p.Kred;
        if (vb_ok) {
            const int tap = col / p.C;
            vb_c = col - tap * p.C;
            vb_e = tap % p.kw;
            const int t2 = tap / p.kw;
            vb_b = t2 % p.kh;
            vb_a = t2 / p.kh;
        }
    }

    auto x_offset = [&](int m, int a, int b, int e, int c, int64_t &off) -> bool {
        const int ow = m % p.Wo;
        int t = m / p.Wo;
        const int oh = t % p.Ho;
        t /= p.Ho;
        const int od = t % p.Do;
        const int n = t / p.Do;
        const int id = od * p.sd - p.pd + a, ih = oh * p.sh - p.ph + b, iw = ow * p.sw - p.pw + e;
        if ((unsigned)id >= (unsigned)p.D || (unsigned)ih >= (unsigned)p.H || (unsigned)iw >= (unsigned)p.W) return false;
        off = ((((int64_t)n * p.D + id) * p.H + ih) * p.W + iw) * p.C + c;
        return true;
    };

    auto fill_rows = [&](int seg0) {
        for (int q = tid; q < SEG; q += NT) {
            const int m = seg0 + q;
            int4 rc = make_int4(-1, 0, 0, 0);
            int64_t rb = 0;
            if (m < mend) {
                const int ow = m % p.Wo;
                int t = m / p.Wo;
                const int oh = t % p.Ho;
                t /= p.Ho;
                const int od = t % p.Do;
                const int n = t / p.Do;
                rc = make_int4(n, od * p.sd - p.pd, oh * p.sh - p.ph, ow * p.sw - p.pw);
                rb = ((((int64_t)n * p.D + rc.y) * p.H + rc.z) * p.W + rc.w) * p.C;
            }
            rowc[q] = rc;
            rowb[q] = rb;
        }
    };
    // per-thread constants of the fast path: its x column as an element offset from a window's
    // first tap, its dy column, and the dy pointer of its first row (advanced by BK rows per step)
    const int64_t tapoff = (((int64_t)vb_a * p.H + vb_b) * p.W + vb_e) * p.C + vb_c;
    const float *acur = p.dy;                          // this thread's dy element of pass 0, current step
    const int64_t astep = (int64_t)(NT / (BM / 4)) * p.K;  // between the rows of consecutive passes
    bool acol_ok = false;
    if (TAB) {
        const int col = k0 + 4 * (tid % (BM / 4));
        acol_ok = col < p.K;
        acur = p.dy + (int64_t)(mbeg + tid / (BM / 4)) * p.K + (acol_ok ? col : 0);
    }
    // (a macro, not a lambda: the prefetch registers av / bv must stay registers)
#define WGRAD_TAB_LOAD(MB)                                                                                                   \
    do {                                                                                                                     \
        _Pragma("unroll") for (int i = 0; i < A_V; ++i)                                                                      \
        {                                                                                                                    \
            const int m = (MB) + (tid + i * NT) / (BM / 4);                                                                  \
            tav[i] = ldg4((acol_ok & (m < mend)) ? acur + i * astep : g_zero4);                                              \
        }                                                                                                                    \
        acur += (int64_t)BK * p.K;                                                                                           \
        _Pragma("unroll") for (int i = 0; i < B_V; ++i)                                                                      \
        {                                                                                                                    \
            const int q = ((MB) - mbeg) % SEG + (tid + i * NT) / (BN / 4);                                                   \
            const int4 rc = rowc[q];                                                                                         \
            const int64_t rb = rowb[q];                                                                                      \
            const bool ok = vb_ok & (rc.x >= 0) & ((unsigned)(rc.y + vb_a) < (unsigned)p.D) &                                \
                            ((unsigned)(rc.z + vb_b) < (unsigned)p.H) & ((unsigned)(rc.w + vb_e) < (unsigned)p.W);           \
            tbv[i] = ldg4(ok ? p.x + (rb + tapoff) : g_zero4);                                                               \
        }                                                                                                                    \
    } while (0)

    auto load_tiles = [&](int mb) {
        if (VECA) {
#pragma unroll
            for (int i = 0; i < A_V; ++i) {
                const int f = tid + i * NT;
                const int m = mb + f / (BM / 4), col = k0 + 4 * (f % (BM / 4));
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (m < mend && col < p.K) v = *reinterpret_cast<const float4 *>(p.dy + (int64_t)m * p.K + col);
                av[i] = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_S; ++i) {
                const int f = tid + i * NT;
                const int m = mb + f / BM, col = k0 + f % BM;
                as[i] = (m < mend && col < p.K) ? p.dy[(int64_t)m * p.K + col] : 0.f;
            }
        }
        if (VECB) {
#pragma unroll
            for (int i = 0; i < B_V; ++i) {
                const int m = mb + (tid + i * NT) / (BN / 4);
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                int64_t off;
                if (vb_ok && m < mend && x_offset(m, vb_a, vb_b, vb_e, vb_c, off))
                    v = *reinterpret_cast<const float4 *>(p.x + off);
                bv[i] = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < B_S; ++i) {
                const int f = tid + i * NT;
                const int m = mb + f / BN, col = j0 + f % BN;
                float v = 0.f;
                if (m < mend && col < p.Kred) {
                    const int tap = col / p.C;
                    const int c = col - tap * p.C;
                    const int e = tap % p.kw;
                    const int t2 = tap / p.kw;
                    int64_t off;
                    if (x_offset(m, t2 / p.kh, t2 % p.kh, e, c, off)) v = p.x[off];
                }
                bs[i] = v;
            }
        }
    };

    auto store_tiles = [&]() {
        if (TAB) return;   // the fast path stores inline (see the main loop)
        if (VECA) {
#pragma unroll
            for (int i = 0; i < A_V; ++i) {
                const int f = tid + i * NT;
                *reinterpret_cast<float4 *>(&As[(f / (BM / 4)) * LDA + 4 * (f % (BM / 4))]) = av[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_S; ++i) {
                const int f = tid + i * NT;
                As[(f / BM) * LDA + f % BM] = as[i];
            }
        }
        if (VECB) {
#pragma unroll
            for (int i = 0; i < B_V; ++i) {
                const int f = tid + i * NT;
                *reinterpret_cast<float4 *>(&Bs[(f / (BN / 4)) * LDB + 4 * (f % (BN / 4))]) = bv[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < B_S; ++i) {
                const int f = tid + i * NT;
                Bs[(f / BN) * LDB + f % BN] = bs[i];
            }
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int lane = tid % 64, wave = tid / 64;
    const int wm = wave / WGN, wn = wave % WGN;
    const int r = lane % 32, h = lane / 32;

    if (TAB) {
        fill_rows(mbeg);
        __syncthreads();
        WGRAD_TAB_LOAD(mbeg);
    } else if (mbeg < mend) {
        load_tiles(mbeg);
    }
    for (int mb = mbeg; mb < mend; mb += BK) {
        store_tiles();
        if (TAB) {
#pragma unroll
            for (int i = 0; i < A_V; ++i) {
                const int f = tid + i * NT;
                *reinterpret_cast<f32x4 *>(&As[(f / (BM / 4)) * LDA + 4 * (f % (BM / 4))]) = tav[i];
            }
#pragma unroll
            for (int i = 0; i < B_V; ++i) {
                const int f = tid + i * NT;
                *reinterpret_cast<f32x4 *>(&Bs[(f / (BN / 4)) * LDB + 4 * (f % (BN / 4))]) = tbv[i];
            }
        }
        // the rows of the next step open a new segment: every load of the old one has been issued
        if (TAB && (mb + BK - mbeg) % SEG == 0) fill_rows(mb + BK);
        __syncthreads();
        if (TAB) WGRAD_TAB_LOAD(mb + BK);   // past the end: every row is marked absent
        else if (mb + BK < mend) load_tiles(mb + BK);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = As[(2 * t + h) * LDA + wm * TM * 32 + i * 32 + r];
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = Bs[(2 * t + h) * LDB + wn * TN * 32 + j * 32 + r];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    float *out = p.out + (int64_t)split * p.K * p.Kred;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = j0 + wn * TN * 32 + j * 32 + r;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + wm * TM * 32 + i * 32 + (v / 4) * 8 + h * 4 + (v % 4);
                if (k < p.K && col < p.Kred) out[(int64_t)k * p.Kred + col] = acc[i][j][v];
            }
        }
}

#undef WGRAD_TAB_LOAD

// dw[e] = sum over splits, in a fixed order: lane group g adds splits g, g+4, g+8, ... and the
// four group sums are combined as ((s0 + s1) + s2) + s3
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float *__restrict__ part, float *__restrict__ dw, int64_t n, int nsplit)
{
    __shared__ float sh[4][64];
    const int l = threadIdx.x % 64, g = threadIdx.x / 64;
    const int64_t e = (int64_t)blockIdx.x * 64 + l;
    float s = 0.f;
    if (e < n) {
#pragma unroll 4
        for (int k = g; k < nsplit; k += 4) s += part[(int64_t)k * n + e];
    }
    sh[g][l] = s;
    __syncthreads();
    if (g == 0 && e < n) dw[e] = ((sh[0][l] + sh[1][l]) + sh[2][l]) + sh[3][l];
}

// ------------------------------------------------------------------ filter gradient, few channels, several taps
//
// For 32 or 64 input and output channels under a 3-wide filter (ResNet-50's 3x3 64 -> 64, the first levels of a
// 3-d CNN) the generic kernel above is bound by what it moves from L2 into LDS, not by the matrix cores: its B
// operand is the im2col view of x, in which every input element appears once per filter tap, and with at most 64
// output channels each staged float feeds at most 128 flops.  Here the taps share what is staged: a workgroup takes
// a segment of P consecutive output pixels of one output row, brings the P x K slice of dy and, for each input row
// (a, b) of its group, the P + 2 input pixels under that segment into LDS once, and its wavefronts -- three sets,
// one per horizontal tap e -- read their B operand from the same LDS row shifted by e pixels.  The reduction index
// of the MFMA is the pixel.  Loads go from global memory straight into LDS (global_load_lds, 16 bytes per lane, no
// staging registers) into a ring of up to four buffers, two or three segments ahead of the one being multiplied
// (one segment ahead left the matrix cores waiting 40 % of the time): one barrier per segment, and a counted wait
// (vmcnt) that lets the younger segments' loads stay in flight.  Each workgroup walks a contiguous range of segments,
// accumulating, and writes one partial K x (its taps) x C block; partials are summed in a fixed order by
// reduce_splits_kernel (deterministic, no atomics).
struct WHaloP {
    const float *dy;   // [M][K]
    const float *x;    // channels-last input
    float *out;        // partials [nsplit][K][Kred]
    int K, C, Kred;
    int N, D, H, W, Do, Ho, Wo;
    int kd, kh, pd, ph, pw;
    int P, PW, PWpad, nseg_w;  // segment length (a multiple of 8), staged input pixels per row (P + 2), its padded LDS extent, segments per output row
    int dy_blocks, row_blocks; // 1 KiB blocks (64 lanes x 16 bytes) of the dy slice and of one input row in LDS
    int lpw;                   // load instructions per wavefront and segment (the same for every wavefront: idle slots load zeros)
    int buf_floats, nbuf;      // LDS floats of one buffer (dy, rows, one block for the idle slots), buffers in the ring
    int nseg;                  // N * Do * Ho * nseg_w
    int seg_per_split, nsplit, groups, total, chunk;
};

typedef __attribute__((address_space(3))) void lds_void_ptr;
typedef __attribute__((address_space(1))) const void glb_void_ptr;

// most load instructions a wavefront issues per segment (its slots' bookkeeping lives in registers)
constexpr int WHALO_MAX_LPW = 4;

// s_waitcnt on the vector-memory counter alone: returns when at most n of this wavefront's loads are outstanding
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    // immediate operand: vmcnt[3:0] | expcnt(7) << 4 | lgkmcnt(15) << 8 | vmcnt[5:4] << 14
    switch (n) {
#define POOCH_VMCNT(N) case N: __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14)); break;
        POOCH_VMCNT(0) POOCH_VMCNT(1) POOCH_VMCNT(2) POOCH_VMCNT(3) POOCH_VMCNT(4) POOCH_VMCNT(5) POOCH_VMCNT(6) POOCH_VMCNT(7) POOCH_VMCNT(8)
#undef POOCH_VMCNT
    default: __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8)); break;   // vmcnt(0)
    }
}


// KB, CB: output / input channels in units of 32; GR: input rows per workgroup.  The GR x KB x CB blocks of 32 x 32
// that belong to one horizontal tap are dealt to GR/GW x KB/IW x CB/JW wavefronts, GW x IW x JW blocks each.
template <int KB, int CB, int GR, int GW, int IW, int JW>
__global__ __launch_bounds__(192 * (GR / GW) * (KB / IW) * (CB / JW)) void wgrad_halo_kernel(WHaloP p)
{
    constexpr int WPT = (GR / GW) * (KB / IW) * (CB / JW), NWV = 3 * WPT;
    constexpr int K = 32 * KB, C = 32 * CB, QK = K / 4, QC = C / 4;
    extern __shared__ __attribute__((aligned(16))) float halo_lds[];

    const int tid = threadIdx.x;
    const int logical = remap_tile(blockIdx.x, p.chunk);
    if (logical >= p.total) return;
    const int split = logical / p.groups, group = logical % p.groups;
    const int lane = tid % 64, wave = __builtin_amdgcn_readfirstlane(tid / 64);   // (uniform: what depends on it stays in scalar registers)
    const int e = wave / WPT, sub = wave % WPT;    // horizontal tap, and which of its blocks
    const int sj = sub % (CB / JW), si = (sub / (CB / JW)) % (KB / IW), sg = sub / ((CB / JW) * (KB / IW));
    const int g0 = sg * GW, i0 = si * IW, j0 = sj * JW;
    const int r = lane % 32, h = lane / 32;

    // a wavefront with a single block alternates between two accumulators (even / odd steps, summed at the end), so
    // that consecutive MFMAs do not depend on each other
    constexpr int SETS = GW * IW * JW == 1 ? 2 : 1;
    f32x16 acc[SETS][GW][IW][JW];
#pragma unroll
    for (int q = 0; q < SETS; ++q)
#pragma unroll
        for (int g = 0; g < GW; ++g)
#pragma unroll
            for (int i = 0; i < IW; ++i)
#pragma unroll
                for (int j = 0; j < JW; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[q][g][i][j][v] = 0.f;

    // This wavefront's load slots: slot k brings block wave + k * NWV of the segment's dy-then-rows sequence of 1 KiB
    // blocks; a slot past the sequence's end loads zeros into the spare block at the end of the buffer, so that every
    // wavefront issues exactly lpw loads per segment and the counted wait below is the same immediate for all.
    // Everything about a slot that does not depend on the segment is worked out here, once: which tensor, where in the
    // buffer, which pixel and channel group this lane brings, which input row (relative to the output row).
    const int x_floats = p.dy_blocks * 256;        // where the input rows start inside a buffer
    int slot_kind[WHALO_MAX_LPW], slot_dst[WHALO_MAX_LPW], slot_da[WHALO_MAX_LPW], slot_db[WHALO_MAX_LPW];   // kind: 0 dy, 1 input row, 2 idle
    int lane_pix[WHALO_MAX_LPW], lane_off[WHALO_MAX_LPW];   // pixel within the segment (dy) or the staged row (x); float offset of the channel group
#pragma unroll
    for (int k = 0; k < WHALO_MAX_LPW; ++k) {
        const int bk = wave + k * NWV;
        slot_kind[k] = 2;
        slot_dst[k] = x_floats + GR * p.PWpad * C;     // the spare block
        slot_da[k] = slot_db[k] = 0;
        lane_pix[k] = lane_off[k] = 0;
        if (bk < p.dy_blocks) {
            const int u = bk * 64 + lane;
            const int pix = u / QK, cpos = u % QK;
            slot_kind[k] = 0;
            slot_dst[k] = bk * 256;
            lane_pix[k] = pix;
            lane_off[k] = 4 * (K == 64 ? cpos ^ ((pix & 1) << 3) : cpos);
        } else if ((bk - p.dy_blocks) / p.row_blocks < GR) {
            const int row = (bk - p.dy_blocks) / p.row_blocks, blk = (bk - p.dy_blocks) % p.row_blocks;
            const int grow = group * GR + row;          // input row (a, b) of this group
            const int u = blk * 64 + lane;
            const int q = u / QC, cpos = u % QC;
            slot_kind[k] = 1;
            slot_dst[k] = x_floats + row * p.PWpad * C + blk * 256;
            slot_da[k] = grow / p.kh - p.pd;
            slot_db[k] = grow % p.kh - p.ph;
            lane_pix[k] = q < p.PW ? q - p.pw : -(1 << 20);   // pieces of the row's padding: never inside the image
            lane_off[k] = 4 * (C == 64 ? cpos ^ ((q & 1) << 3) : cpos);
        }
    }

    const int seg_beg = split * p.seg_per_split;
    const int seg_end = min(p.nseg, seg_beg + p.seg_per_split);
    // coordinates of the segment whose loads are issued next; stepped with carries
    int wseg = seg_beg % p.nseg_w;
    int t0 = seg_beg / p.nseg_w;
    int oh = t0 % p.Ho;
    t0 /= p.Ho;
    int od = t0 % p.Do;
    int n = t0 / p.Do;

    // Position c (16 bytes) of pixel q's row in LDS holds channel group c ^ swz(q): for 64-float rows the two halves swap
    // on odd pixels, so that the two pixels a wavefront reads at once (lane halves h = 0, 1) sit in different banks.
    // The swap is applied to the source address: a lane's LDS position is fixed by global_load_lds (base + 16 * lane).
    auto issue = [&](int buf) {
        float *const base_s = halo_lds + buf * p.buf_floats;
        const int w0 = wseg * p.P;
        const int pv = min(p.P, p.Wo - w0);        // pixels of the segment that exist
        const int64_t m0 = (((int64_t)n * p.Do + od) * p.Ho + oh) * p.Wo + w0;
#pragma unroll
        for (int k = 0; k < WHALO_MAX_LPW; ++k) {
            if (k < p.lpw) {
                const float *src = g_zero4;
                if (slot_kind[k] == 0) {
                    if (lane_pix[k] < pv) src = p.dy + ((m0 + lane_pix[k]) * K + lane_off[k]);
                } else if (slot_kind[k] == 1) {
                    const int id = od + slot_da[k], ih = oh + slot_db[k], iw = w0 + lane_pix[k];
                    const bool ok = ((unsigned)id < (unsigned)p.D) & ((unsigned)ih < (unsigned)p.H) & ((unsigned)iw < (unsigned)p.W);
                    if (ok) src = p.x + (((((int64_t)n * p.D + id) * p.H + ih) * p.W + iw) * C + lane_off[k]);
                }
                __builtin_amdgcn_global_load_lds((glb_void_ptr *)src, (lds_void_ptr *)(base_s + slot_dst[k]), 16, 0, 0);
            }
        }
        if (++wseg == p.nseg_w) {
            wseg = 0;
            if (++oh == p.Ho) {
                oh = 0;
                if (++od == p.Do) {
                    od = 0;
                    ++n;
                }
            }
        }
    };

    const int ahead = p.nbuf - 1;                  // segments in flight beyond the one being multiplied
    for (int k = 0; k < ahead; ++k)
        if (seg_beg + k < seg_end) issue(k);
    int buf = 0;
    for (int sgm = seg_beg; sgm < seg_end; ++sgm) {
        // loads are retired in order: segment sgm's have landed once only the younger segments' are outstanding
        wait_vmcnt_at_most(min(ahead - 1, seg_end - 1 - sgm) * p.lpw);
        // A bare barrier: everyone's loads of segment sgm have landed, and everyone has finished reading the previous
        // buffer (its fragments were consumed by MFMAs already issued).  __syncthreads() would not do: its fence makes
        // the compiler wait for every outstanding load, the younger segments' too, which is the latency the ring hides.
        // The empty asm statements keep the compiler from moving LDS reads or loads across the barrier.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // The next loads (into the buffer multiplied last) are issued from inside the step loop, at a step that depends
        // on the wavefront: right after the barrier every wavefront would run that address arithmetic at the same time
        // and the matrix cores would sit idle meanwhile; staggered, it runs under the other wavefronts' MFMAs.
        const bool more = sgm + ahead < seg_end;
        const int issue_buf = buf == 0 ? p.nbuf - 1 : buf - 1;
        const float *const dy_s = halo_lds + buf * p.buf_floats;
        const float *const x_s = dy_s + x_floats;
        // MFMA step t multiplies pixels 2t and 2t + 1 (lane half h takes pixel 2t + h)
        const int steps = p.P / 2;
        const float *ap = dy_s + h * K + r;
        const float *bp = x_s + (h + e) * C + r;
        const int hs = K == 64 ? (h << 5) : 0, qs = C == 64 ? (((h + e) & 1) << 5) : 0;   // bank swap of this lane's pixels (their parity is fixed: they advance by two)
        float af0[2][IW], bf0[2][GW][JW], af1[2][IW], bf1[2][GW][JW], af2[2][IW], bf2[2][GW][JW], af3[2][IW], bf3[2][GW][JW];
        auto load_pair = [&](float (&af)[2][IW], float (&bf)[2][GW][JW], int t) {
#pragma unroll
            for (int d = 0; d < 2; ++d) {
#pragma unroll
                for (int i = 0; i < IW; ++i) af[d][i] = ap[2 * (t + d) * K + (((i0 + i) * 32) ^ hs)];
#pragma unroll
                for (int g = 0; g < GW; ++g)
#pragma unroll
                    for (int j = 0; j < JW; ++j) bf[d][g][j] = bp[((g0 + g) * p.PWpad + 2 * (t + d)) * C + (((j0 + j) * 32) ^ qs)];
            }
        };
        auto mul_pair = [&](const float (&af)[2][IW], const float (&bf)[2][GW][JW]) {
#pragma unroll
            for (int d = 0; d < 2; ++d)
#pragma unroll
                for (int g = 0; g < GW; ++g)
#pragma unroll
                    for (int i = 0; i < IW; ++i)
#pragma unroll
                        for (int j = 0; j < JW; ++j)
                            acc[d % SETS][g][i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[d][i], bf[d][g][j], acc[d % SETS][g][i][j], 0, 0, 0);
        };
        // one MFMA, then its share of the LDS reads issued in the same stretch of code
        constexpr int NM = 2 * GW * IW * JW, NR = 2 * (IW + GW * JW), RPM = (NR + NM - 1) / NM;
        auto interleave = [&]() {
#pragma unroll
            for (int q = 0; q < NM; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);   // LDS reads
            }
        };
        // Pairs of steps go round four sets of fragment registers: while pair k is multiplied, pair k + 2 is read from
        // LDS, so a read has two pairs' MFMAs to arrive in.  Four pairs per trip; P is a multiple of 8, so what is left
        // after the last whole trip is nothing or two pairs, which are in their registers by then.  Loads past the end
        // fetch a pair that exists and is not used.
        const int last = steps - 2;
        const int issue_at = 8 * ((wave / 4) % 3);     // the three wavefronts of a SIMD take turns
        load_pair(af0, bf0, 0);
        load_pair(af1, bf1, 2);
        int t = 0;
        for (; t + 8 <= steps; t += 8) {
            if (more && t == issue_at) issue(issue_buf);
            load_pair(af2, bf2, min(t + 4, last));
            mul_pair(af0, bf0);
            interleave();
            load_pair(af3, bf3, min(t + 6, last));
            mul_pair(af1, bf1);
            interleave();
            load_pair(af0, bf0, min(t + 8, last));
            mul_pair(af2, bf2);
            interleave();
            load_pair(af1, bf1, min(t + 10, last));
            mul_pair(af3, bf3);
            interleave();
        }
        if (more && issue_at >= t) issue(issue_buf);   // (a segment shorter than the wavefront's turn)
        if (t < steps) {
            mul_pair(af0, bf0);
            mul_pair(af1, bf1);
        }
        buf = buf + 1 == p.nbuf ? 0 : buf + 1;
    }
    wait_vmcnt_at_most(0);

    float *out = p.out + (int64_t)split * p.K * p.Kred;
#pragma unroll
    for (int g = 0; g < GW; ++g) {
        const int tap = (group * GR + g0 + g) * 3 + e;
#pragma unroll
        for (int i = 0; i < IW; ++i)
#pragma unroll
            for (int j = 0; j < JW; ++j) {
                const int col = tap * C + (j0 + j) * 32 + r;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = (i0 + i) * 32 + (v / 4) * 8 + h * 4 + (v % 4);
                    out[(int64_t)k * p.Kred + col] = SETS == 2 ? acc[0][g][i][j][v] + acc[SETS - 1][g][i][j][v] : acc[0][g][i][j][v];
                }
            }
    }
}

// ---- filter gradient of that first layer: one live input channel, 32 output channels, 3 x 3 x 3 ----------------------------
// dw[k][tap] = sum over positions of dy[pos][k] * x[pos + tap]: 27 x 32 results from 0.9 GB of dy on a 192^3 volume.  As a
// GEMM over the four stored channels the generic kernel stages an im2col view (a 108-wide B operand, three quarters of
// it zeros) and needs 0.93 ms; the work is reading dy once.  Here every WAVE walks bricks of 2 x 8 x 8 positions on its
// own -- no workgroup barrier until the end: it loads the brick's 128 rows of dy straight into registers (lanes 0 - 31
// one row, lanes 32 - 63 the next: whole 128-byte rows), keeps the brick's 4 x 10 x 10 input values in its private 1.6 KB
// of LDS and gathers from there.  One MFMA per pair of positions (the reduction index is the position): A = dy (index =
// output channel), B = the input value under tap (lane % 32).  The eight waves of a workgroup add their blocks in a
// fixed order at the end and write one partial [32][27][Cs] (zeros in the dead channels); reduce_splits_kernel adds the
// partials in a fixed order.
struct WGradC1P {
    const float *dy, *x;
    float *out;              // [nsplit][32][27][Cs]
    int N, D, H, W, Cs;
    int bricks, per_wave;    // bricks in all, bricks per wave (wave g of the grid takes [g * per_wave, (g + 1) * per_wave))
};

__global__ __launch_bounds__(512) void wgrad3_c1_kernel(WGradC1P p)
{
    __shared__ __attribute__((aligned(16))) float lds[8 * 1024];     // per wave: the halo (400 floats); at the end: its 32 x 32 block
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    float *halo = lds + wave * 1024;
    const int D = p.D, H = p.H, W = p.W, CS = p.Cs;
    const int nbw = W / C3_BW, nbh = H / C3_BH, nbd = D / C3_BD;
    // B operand of lane (r, h) at step s of a line: halo[(line base) + 2 s + h + off], off = the tap's offset in the halo
    const int tap = r < 27 ? r : 26;                                  // (columns 27 .. 31 of the block are not stored)
    const int boff = ((tap / 9) * C3_HH + (tap / 3) % 3) * C3_HW + tap % 3 + h;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const int g = blockIdx.x * 8 + wave;
    const int b_end = min((g + 1) * p.per_wave, p.bricks);
    for (int b = g * p.per_wave; b < b_end; ++b) {                    // (wave-uniform bounds)
        int t = b;
        const int w0 = (t % nbw) * C3_BW; t /= nbw;
        const int h0 = (t % nbh) * C3_BH; t /= nbh;
        const int d0 = (t % nbd) * C3_BD;
        const int n = t / nbd;
        // the brick's dy: 16 lines (d, h) of 8 positions = 1 KB each; step s of a line covers positions 2 s and 2 s + 1
        float a[64];
#pragma unroll
        for (int line = 0; line < 16; ++line) {
            const int64_t m = (((int64_t)n * D + d0 + line / 8) * H + h0 + line % 8) * W + w0;
            const float *dp = p.dy + m * C3_C + lane;
#pragma unroll
            for (int s = 0; s < 4; ++s) a[line * 4 + s] = ldg1(dp + s * 64);
        }
        const float *x = p.x + (int64_t)n * D * H * W * CS;
#pragma unroll
        for (int k = 0; k < 7; ++k) {
            const int u = lane + 64 * k;
            const int id = d0 + u / (C3_HH * C3_HW) - 1, ih = h0 + (u / C3_HW) % C3_HH - 1, iw = w0 + u % C3_HW - 1;
            const bool ok = u < C3_NPIX && (unsigned)id < (unsigned)D && (unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W;
            const float v = ok ? ldg1(x + (((int64_t)id * H + ih) * W + iw) * CS) : 0.f;
            if (u < C3_NPIX) halo[u] = v;
        }
        // (LDS serves a wave's instructions in order: its own reads below see these writes, and the next brick's writes
        // come after this brick's reads; the wave barrier emits no instruction, it only keeps the compiler from moving
        // LDS accesses across it)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int line = 0; line < 16; ++line) {
            const float *hp = halo + ((line / 8) * C3_HH + line % 8) * C3_HW + boff;
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[line * 4 + s], hp[2 * s], acc, 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();
    }
    // element v of lane (r, h): output channel 8 * (v / 4) + 4 * h + v % 4, tap r
    __syncthreads();
    float *mine = lds + wave * 1024;
#pragma unroll
    for (int v = 0; v < 16; ++v) mine[(8 * (v / 4) + 4 * h + v % 4) * 32 + r] = acc[v];
    __syncthreads();
    float *out = p.out + (int64_t)blockIdx.x * 32 * 27 * CS;
    for (int e = tid; e < 32 * 27 * CS; e += 512) {
        const int c = e % CS, kt = e / CS, tp = kt % 27, k = kt / 27;
        float v = 0.f;
        if (c == 0) {
            v = lds[k * 32 + tp];
#pragma unroll
            for (int w2 = 1; w2 < 8; ++w2) v += lds[w2 * 1024 + k * 32 + tp];
        }
        out[e] = v;
    }
}

struct WGradC1Cfg {
    bool use;
    int nsplit, per_wave, bricks;
};

WGradC1Cfg wgrad3_c1_cfg(const ConvGeom &g)
{
    static const bool off = getenv("POOCH_NO_CONV3_C1") != nullptr;
    WGradC1Cfg c{false, 0, 0, 0};
    if (off || g.Clive != 1 || g.K != C3_C || g.kd != 3 || g.kh != 3 || g.kw != 3) return c;
    if (g.sd != 1 || g.sh != 1 || g.sw != 1 || g.pd != 1 || g.ph != 1 || g.pw != 1) return c;
    if (g.Do != g.D || g.Ho != g.H || g.Wo != g.W || g.D % C3_BD != 0 || g.H % C3_BH != 0 || g.W % C3_BW != 0) return c;
    c.bricks = (int)(g.rows_out() / (C3_BD * C3_BH * C3_BW));
    if (c.bricks < 1) return c;
    // one workgroup of eight waves per compute unit where there is that much work, at least four bricks per wave
    c.nsplit = (c.bricks + 31) / 32;
    if (c.nsplit > NCU) c.nsplit = NCU;
    c.per_wave = (c.bricks + c.nsplit * 8 - 1) / (c.nsplit * 8);
    c.nsplit = (c.bricks + c.per_wave * 8 - 1) / (c.per_wave * 8);     // no workgroup without bricks
    c.use = true;
    return c;
}

// ---- filter gradient, 3 x 3 x 3, 32 or 64 channels on either side, whole bricks: brick and halo resident in LDS ------------
// wgrad_halo_kernel walks segments of one output row: a barrier per segment of at most 64 positions, 32 MFMAs per wave between
// two barriers, and three groups of workgroups (one per depth tap) that each stage dy and the input rows again (6.6 GB moved for
// 1.8 GB of operands at 192^3, matrix pipe busy 61 %).  Here a workgroup of four waves takes a brick of 2 x 8 x 8 positions:
// the brick's dy rows (128 x 32) and the 4 x 10 x 10 input positions under its 27 taps go to LDS once (76 KB, two workgroups
// per CU, which load and multiply in turns as those of conv3_halo_kernel do); wave w multiplies the taps 7 w .. 7 w + 6 (the
// fourth wave's seventh is a repeat whose result is dropped: uniform code): per line of eight positions four reads of dy (A
// operand: index = output channel, reduction index = position) and 28 of the input (B operand: index = input channel) for 28
// MFMAs -- 448 per wave between two barriers.  Workgroups are persistent (exactly as many as are resident), each accumulates
// over a contiguous range of bricks and writes one partial [32][27][32] straight from its registers; reduce_splits_kernel
// adds the partials in a fixed order.  With 64 channels on a side the result falls into two or four such 32 x 27 x 32 blocks
// (kq, cq), each the work of a workgroup of its own that stages only its 32 channels of dy and of the input (so the LDS
// footprint stays at 76 KB; dy and the input are then read twice, from the L2 for the most part).
constexpr size_t WGRAD3_BRICK_LDS = (size_t)(C3_NPIX + C3_BD * C3_BH * C3_BW) * C3_LP * sizeof(float);   // 76 KB

struct WGradB3P {
    const float *dy, *x;
    float *out;              // [splits][K][27][C]
    int N, D, H, W;
    int K, C;                // 32 or 64 each: a workgroup computes one 32 x 27 x 32 block (kq, cq) of the result for its bricks
    int bricks, per_split;   // split g takes bricks [g * per_split, min(bricks, (g + 1) * per_split)); workgroup = (g, kq, cq)
};

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void wgrad3_brick_kernel(WGradB3P p)
{
    extern __shared__ __attribute__((aligned(16))) float brick_lds[];        // WGRAD3_BRICK_LDS bytes
    float *xs = brick_lds, *dys = brick_lds + C3_NPIX * C3_LP;
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int D = p.D, H = p.H, W = p.W, KT = p.K, CT = p.C;
    const int nbw = W / C3_BW, nbh = H / C3_BH, nbd = D / C3_BD;
    const int nsub = (KT / 32) * (CT / 32), sub = blockIdx.x % nsub, split = blockIdx.x / nsub;
    const int k0 = 32 * (sub / (CT / 32)), c0 = 32 * (sub % (CT / 32));
    f32x16 acc[7];
#pragma unroll
    for (int i = 0; i < 7; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    int toff[7];                                                              // halo offset (in pixels) of this wave's taps
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        const int tap = min(7 * wave + i, 26);
        toff[i] = ((tap / 9) * C3_HH + (tap / 3) % 3) * C3_HW + tap % 3;
    }
    const float *arow = dys + h * C3_LP + r;                                  // + (8 line + 2 s) * C3_LP
    const float *brow = xs + h * C3_LP + r;                                   // + (line's pixel + tap offset + 2 s) * C3_LP
    const int b_end = min((split + 1) * p.per_split, p.bricks);
    for (int b = split * p.per_split; b < b_end; ++b) {
        int t = b;
        const int w0 = (t % nbw) * C3_BW; t /= nbw;
        const int h0 = (t % nbh) * C3_BH; t /= nbh;
        const int d0 = (t % nbd) * C3_BD;
        const int n = t / nbd;
        __syncthreads();                                  // the previous brick has been read
        {
            // input halo: line (pd, ph) = 10 pixels x 32 of their channels = 80 lanes x 16 bytes; wave w takes lines w, w + 4, ...
            // (wave-uniform); dy: 16 lines of 8 positions x 32 of their channels = 64 lanes x 16 bytes, wave w takes lines w, w + 4, ...
            const float *x = p.x + (int64_t)n * D * H * W * CT + c0;
            constexpr int NL = C3_HD * C3_HH / 4;
            f32x4 v0[NL], v1[NL], vd[4];
            const int pw0 = lane / 8, q4 = 4 * (lane % 8);
            const int lx = pw0 * CT + q4, ly = pw0 * KT + q4;     // this lane's 16 bytes of a line: pixel pw0, channels q4 .. q4 + 3
            const bool in0 = !(w0 == 0 && pw0 == 0);
            const bool in1 = lane < 16 && !(w0 + C3_BW == W && pw0 == 1);
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                const int line = wave + 4 * k, pd = line / C3_HH, ph = line % C3_HH;
                const int id = d0 + pd - 1, ih = h0 + ph - 1;
                const bool lok = (unsigned)id < (unsigned)D && (unsigned)ih < (unsigned)H;
                const float *src = x + ((((int64_t)(lok ? id : 0) * H + (lok ? ih : 0)) * W + w0) * CT - CT);
                v0[k] = (lok && in0) ? ldg4(src + lx) : z;
                v1[k] = (lok && in1) ? ldg4(src + lx + 8 * CT) : z;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int line = wave + 4 * k;
                const int64_t m = (((int64_t)n * D + d0 + line / 8) * H + h0 + line % 8) * W + w0;
                vd[k] = ldg4(p.dy + m * KT + k0 + ly);
            }
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                const int line = wave + 4 * k;
                float *dst = xs + (line * C3_HW + pw0) * C3_LP + q4;
                *reinterpret_cast<f32x4 *>(dst) = v0[k];
                if (lane < 16) *reinterpret_cast<f32x4 *>(dst + 8 * C3_LP) = v1[k];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int line = wave + 4 * k;
                *reinterpret_cast<f32x4 *>(dys + (line * 8 + pw0) * C3_LP + q4) = vd[k];
            }
        }
        __syncthreads();
        // operands of line l + 1 are read before the MFMAs of line l (the fences keep the compiler from sinking the reads)
        float a0[4], b0[7][4], a1[4], b1[7][4];
        auto load = [&](float (&a)[4], float (&bb)[7][4], int line) {
            const float *ap = arow + line * 8 * C3_LP;
            const float *bp = brow + ((line / 8) * C3_HH + line % 8) * C3_HW * C3_LP;
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) a[s2] = ap[2 * s2 * C3_LP];
#pragma unroll
            for (int i = 0; i < 7; ++i)
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) bb[i][s2] = bp[(toff[i] + 2 * s2) * C3_LP];
        };
        auto mul = [&](const float (&a)[4], const float (&bb)[7][4]) {
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
                for (int i = 0; i < 7; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s2], bb[i][s2], acc[i], 0, 0, 0);
        };
        load(a0, b0, 0);
#pragma unroll 1
        for (int line = 0; line < 14; line += 2) {
            load(a1, b1, line + 1);
            __builtin_amdgcn_sched_barrier(0);
            mul(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            load(a0, b0, line + 2);
            __builtin_amdgcn_sched_barrier(0);
            mul(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        load(a1, b1, 15);
        __builtin_amdgcn_sched_barrier(0);
        mul(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        mul(a1, b1);
    }
    // element v of lane (r, h): output channel 8 * (v / 4) + 4 * h + v % 4, input channel r
    float *out = p.out + ((int64_t)split * KT + k0) * 27 * CT + c0;
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        const int tap = 7 * wave + i;
        if (tap < 27) {
#pragma unroll
            for (int v = 0; v < 16; ++v) out[((8 * (v / 4) + 4 * h + v % 4) * 27 + tap) * CT + r] = acc[i][v];
        }
    }
}

struct WGradB3Cfg {
    bool use;
    int nsplit, per_split, bricks;   // splits of the brick range (each split: one workgroup per 32 x 27 x 32 block of the result)
};

WGradB3Cfg wgrad3_brick_cfg(const ConvGeom &g)
{
    static const bool off = getenv("POOCH_NO_WGRAD3_BRICK") != nullptr;
    WGradB3Cfg c{false, 0, 0, 0};
    if (off || g.C % 32 != 0 || g.K % 32 != 0 || g.C > 256 || g.K > 256 || g.kd != 3 || g.kh != 3 || g.kw != 3) return c;
    if (g.sd != 1 || g.sh != 1 || g.sw != 1 || g.pd != 1 || g.ph != 1 || g.pw != 1) return c;
    if (g.Do != g.D || g.Ho != g.H || g.Wo != g.W || g.D % C3_BD != 0 || g.H % C3_BH != 0 || g.W % C3_BW != 0) return c;
    c.bricks = (int)(g.rows_out() / (C3_BD * C3_BH * C3_BW));
    if (c.bricks < 1) return c;
    const int nsub = (g.K / 32) * (g.C / 32);
    c.nsplit = 2 * NCU / nsub;                                       // as many workgroups as are resident at once
    if (c.nsplit > c.bricks) c.nsplit = c.bricks;
    c.per_split = (c.bricks + c.nsplit - 1) / c.nsplit;
    c.nsplit = (c.bricks + c.per_split - 1) / c.per_split;           // none without bricks
    c.use = true;
    return c;
}

// ---- filter gradient of the stem: dw[n][tap][c] = sum over output positions of dy[pos][n] * x[2 pos - 3 + tap][c] -----------
// The generic kernel stages an im2col view of the four stored channels (a 196-wide B operand for 147 live values) and runs
// at 60 TFLOP/s of live flops (2.5 ms at batch 640).  Here the tile's input patch sits in LDS as in stem7_fwd_kernel; a
// wave takes two of the tile's eight rows (16 pairs of positions: the reduction index of the MFMA is the position), reads
// the pair's dy rows straight from global memory (A operand: index = output channel, two blocks of 32) and gathers the B
// operand (index = reduction value k = 3 tap + c, five blocks of 32 for 147 values) from the patch at a per-lane offset: ten
// accumulator blocks per wave, ten MFMAs per pair for two loads and five gathers.  dy for the NEXT tile is loaded into the
// registers a pair has just been multiplied from.  Persistent workgroups; at the end the four waves' blocks are added in
// a fixed order through LDS into one partial [64][49][4] per workgroup (zeros in the dead channel), and
// reduce_splits_kernel adds the partials in a fixed order.
struct Stem7WP {
    const float *dy, *x;
    float *out;              // [workgroups][64][49][4]
    int N, H, W, Ho, Wo;
    int tiles, per_wg;
};

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void stem7_wgrad_kernel(Stem7WP p)
{
    __shared__ __attribute__((aligned(16))) float patch[S7_PATCH];
    __shared__ __attribute__((aligned(16))) float red[4 * 1024];
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int Ho = p.Ho, Wo = p.Wo, H = p.H, W = p.W;
    const int tw = Wo / S7_TW, th = Ho / S7_TH;
    f32x16 acc[2][5];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 5; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    // B operand of lane (r, h), block jb, pair s: patch[(2 (2 wave + s / 8)) * S7_RS + 2 (s % 8) + h + s7_off(32 jb + r)]
    const float *bptr[5];
#pragma unroll
    for (int jb = 0; jb < 5; ++jb) bptr[jb] = patch + (4 * wave) * S7_RS + h + s7_off(min(32 * jb + r, 147));
    constexpr int NPF = (S7_PH * S7_PW + 255) / 256;
    f32x4 pf[NPF];
    float a0[16], a1[16];                                // dy of the tile's pairs: channels r and 32 + r of position 2 s + h
    auto fetch = [&](int tile) {
        int t = tile;
        const int ox0 = (t % tw) * S7_TW; t /= tw;
        const int oy0 = (t % th) * S7_TH;
        const float *x = p.x + (int64_t)(t / th) * H * W * 4;
#pragma unroll
        for (int j = 0; j < NPF; ++j) {
            const int u = tid + 256 * j, py = u / S7_PW, px = u % S7_PW;
            const int iy = 2 * oy0 - 3 + py, ix = 2 * ox0 - 3 + px;
            const bool ok = u < S7_PH * S7_PW && (unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            pf[j] = ok ? ldg4(x + ((int64_t)iy * W + ix) * 4) : z;
        }
    };
    auto dyrow = [&](int tile, int s) -> const float * {
        int t = tile;
        const int ox0 = (t % tw) * S7_TW; t /= tw;
        const int oy0 = (t % th) * S7_TH;
        const int n = t / th;
        const int64_t m = ((int64_t)n * Ho + oy0 + 2 * wave + s / 8) * Wo + ox0 + 2 * (s % 8) + h;
        return p.dy + m * 64 + r;
    };
    const int t_beg = blockIdx.x * p.per_wg, t_end = min(t_beg + p.per_wg, p.tiles);
    if (t_beg < t_end) {
        fetch(t_beg);
#pragma unroll
        for (int s2 = 0; s2 < 16; ++s2) {
            const float *dp = dyrow(t_beg, s2);
            a0[s2] = ldg1(dp);
            a1[s2] = ldg1(dp + 32);
        }
    }
    for (int tile = t_beg; tile < t_end; ++tile) {
        __syncthreads();                                  // the previous tile's patch has been read
#pragma unroll
        for (int j = 0; j < NPF; ++j) {
            const int u = tid + 256 * j, py = u / S7_PW, px = u % S7_PW;
            if (u < S7_PH * S7_PW) {
                float *d = patch + ((px & 1) * S7_PH + py) * S7_RS + (px >> 1);
                d[0] = pf[j].x;
                d[2 * S7_PH * S7_RS] = pf[j].y;
                d[4 * S7_PH * S7_RS] = pf[j].z;
            }
        }
        __syncthreads();
        const int next = min(tile + 1, t_end - 1);        // (the last tile again: no branch around the loads)
        fetch(next);
#pragma unroll
        for (int s2 = 0; s2 < 16; ++s2) {
            const int so = (2 * (s2 / 8)) * S7_RS + 2 * (s2 % 8);
#pragma unroll
            for (int jb = 0; jb < 5; ++jb) {
                const float bv = bptr[jb][so];
                acc[0][jb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[s2], bv, acc[0][jb], 0, 0, 0);
                acc[1][jb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s2], bv, acc[1][jb], 0, 0, 0);
            }
            const float *dp = dyrow(next, s2);
            a0[s2] = ldg1(dp);
            a1[s2] = ldg1(dp + 32);
        }
    }
    // element v of lane (r, h) of block (nb, jb): output channel 32 nb + 8 (v / 4) + 4 h + v % 4, reduction value 32 jb + r
    float *out = p.out + (int64_t)blockIdx.x * 64 * 49 * 4;
    for (int e = tid; e < 64 * 49; e += 256) out[4 * e + 3] = 0.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int jb = 0; jb < 5; ++jb) {
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave * 1024 + (8 * (v / 4) + 4 * h + v % 4) * 32 + r] = acc[nb][jb][v];
            __syncthreads();
            for (int e = tid; e < 1024; e += 256) {
                const int k = 32 * jb + e % 32, n = 32 * nb + e / 32;
                if (k < 147) out[(n * 49 + k / 3) * 4 + k % 3] = ((red[e] + red[1024 + e]) + red[2048 + e]) + red[3072 + e];
            }
        }
}

struct Stem7WCfg {
    bool use;
    int nsplit, per_wg, tiles;
};

Stem7WCfg stem7_wgrad_cfg(const ConvGeom &g)
{
    static const bool off = getenv("POOCH_NO_STEM7") != nullptr;
    Stem7WCfg c{false, 0, 0, 0};
    if (off || g.Clive != 3 || g.C != 4 || g.K != 64 || g.D != 1 || g.kd != 1 || g.kh != 7 || g.kw != 7) return c;
    if (g.sd != 1 || g.sh != 2 || g.sw != 2 || g.pd != 0 || g.ph != 3 || g.pw != 3) return c;
    if (g.H != 2 * g.Ho || g.W != 2 * g.Wo || g.Ho % S7_TH != 0 || g.Wo % S7_TW != 0) return c;
    c.tiles = (int)(g.rows_out() / (S7_TH * S7_TW));
    if (c.tiles < 1) return c;
    c.nsplit = c.tiles < 2 * NCU ? c.tiles : 2 * NCU;                // as many workgroups as are resident at once
    c.per_wg = (c.tiles + c.nsplit - 1) / c.nsplit;
    c.nsplit = (c.tiles + c.per_wg - 1) / c.per_wg;
    c.use = true;
    return c;
}

// ---- filter gradient, 3 x 3 (2-d), multiples of 32 channels, whole 8 x 8 bricks: two images' bricks and halos in LDS -------
// The same scheme for ResNet-50's 3 x 3 layers at 56 x 56 (64 -> 64: wgrad_halo_kernel 97 TFLOP/s in the step).  Nine taps do not
// divide over four waves, so here the waves split the POSITIONS: a workgroup takes the 8 x 8 brick at the same place of two
// consecutive images (128 positions, 16 lines of 8; halo 2 x 10 x 10 pixels; 47 KB of LDS), wave w multiplies the lines
// 4 w .. 4 w + 3 under all nine taps -- nine accumulator blocks per wave; per line 4 reads of dy and 27 of the input (three
// halo rows of nine pixels) for 36 MFMAs -- and the four waves' blocks are added in a fixed order through LDS at the end.
// Persistent workgroups, one partial [K][9][C] per split, blocks of 32 x 9 x 32 as in wgrad3_brick_kernel.
constexpr int W2_NPIX = 2 * C3_HH * C3_HW;

struct WGradB2P {
    const float *dy, *x;
    float *out;              // [splits][K][9][C]
    int N, H, W;
    int K, C;
    int bricks, per_split;   // bricks = (N / 2) * (H / 8) * (W / 8)
};

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void wgrad2_brick_kernel(WGradB2P p)
{
    __shared__ __attribute__((aligned(16))) float lds2[(W2_NPIX + 128) * C3_LP];
    float *xs = lds2, *dys = lds2 + W2_NPIX * C3_LP;
    const int tid = threadIdx.x, lane = tid % 64, r = lane % 32, h = lane / 32;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int H = p.H, W = p.W, KT = p.K, CT = p.C;
    const int nbw = W / C3_BW, nbh = H / C3_BH;
    const int nsub = (KT / 32) * (CT / 32), sub = blockIdx.x % nsub, split = blockIdx.x / nsub;
    const int k0 = 32 * (sub / (CT / 32)), c0 = 32 * (sub % (CT / 32));
    f32x16 acc[9];
#pragma unroll
    for (int i = 0; i < 9; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float *arow = dys + h * C3_LP + r;                                  // + (8 line + 2 s) * C3_LP
    const float *brow = xs + h * C3_LP + r;                                   // + ((image * 10 + row + tb) * 10 + j) * C3_LP
    const int b_end = min((split + 1) * p.per_split, p.bricks);
    for (int b = split * p.per_split; b < b_end; ++b) {
        int t = b;
        const int w0 = (t % nbw) * C3_BW; t /= nbw;
        const int h0 = (t % nbh) * C3_BH;
        const int n0 = 2 * (t / nbh);
        __syncthreads();                                  // the previous bricks have been read
        {
            // input halo: 20 lines (image, ph) of 10 pixels x 32 of their channels = 80 lanes x 16 bytes, wave w takes lines
            // w, w + 4, ...; dy: 16 lines of 8 positions x 32 of their channels, wave w takes lines w, w + 4, ...
            constexpr int NL = 2 * C3_HH / 4;
            f32x4 v0[NL], v1[NL], vd[4];
            const int pw0 = lane / 8, q4 = 4 * (lane % 8);
            const int lx = pw0 * CT + q4, ly = pw0 * KT + q4;
            const bool in0 = !(w0 == 0 && pw0 == 0);
            const bool in1 = lane < 16 && !(w0 + C3_BW == W && pw0 == 1);
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                const int line = wave + 4 * k, img = line / C3_HH, ph = line % C3_HH;
                const int ih = h0 + ph - 1;
                const bool lok = (unsigned)ih < (unsigned)H;
                const float *src = p.x + ((((int64_t)(n0 + img) * H + (lok ? ih : 0)) * W + w0) * CT - CT) + c0;
                v0[k] = (lok && in0) ? ldg4(src + lx) : z;
                v1[k] = (lok && in1) ? ldg4(src + lx + 8 * CT) : z;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int line = wave + 4 * k;
                const int64_t m = (((int64_t)(n0 + line / 8)) * H + h0 + line % 8) * W + w0;
                vd[k] = ldg4(p.dy + m * KT + k0 + ly);
            }
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                const int line = wave + 4 * k;
                float *dst = xs + (line * C3_HW + pw0) * C3_LP + q4;
                *reinterpret_cast<f32x4 *>(dst) = v0[k];
                if (lane < 16) *reinterpret_cast<f32x4 *>(dst + 8 * C3_LP) = v1[k];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int line = wave + 4 * k;
                *reinterpret_cast<f32x4 *>(dys + (line * 8 + pw0) * C3_LP + q4) = vd[k];
            }
        }
        __syncthreads();
        // this wave's four lines; operands of the next line are read before the MFMAs of the current one
        float a0[4], b0[3][9], a1[4], b1[3][9];
        auto load = [&](float (&a)[4], float (&bb)[3][9], int line) {
            const float *ap = arow + line * 8 * C3_LP;
            const float *bp = brow + ((line / 8) * C3_HH + line % 8) * C3_HW * C3_LP;
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) a[s2] = ap[2 * s2 * C3_LP];
#pragma unroll
            for (int tb = 0; tb < 3; ++tb)
#pragma unroll
                for (int j = 0; j < 9; ++j) bb[tb][j] = bp[(tb * C3_HW + j) * C3_LP];
        };
        auto mul = [&](const float (&a)[4], const float (&bb)[3][9]) {
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
                for (int tb = 0; tb < 3; ++tb)
#pragma unroll
                    for (int te = 0; te < 3; ++te)
                        acc[tb * 3 + te] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s2], bb[tb][2 * s2 + te], acc[tb * 3 + te], 0, 0, 0);
        };
        const int l0 = 4 * wave;
        load(a0, b0, l0);
        load(a1, b1, l0 + 1);
        __builtin_amdgcn_sched_barrier(0);
        mul(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        load(a0, b0, l0 + 2);
        __builtin_amdgcn_sched_barrier(0);
        mul(a1, b1);
        __builtin_amdgcn_sched_barrier(0);
        load(a1, b1, l0 + 3);
        __builtin_amdgcn_sched_barrier(0);
        mul(a0, b0);
        __builtin_amdgcn_sched_barrier(0);
        mul(a1, b1);
    }
    // element v of lane (r, h) of block tap: output channel 8 * (v / 4) + 4 * h + v % 4, input channel r; the four waves' blocks
    // are added in wave order
    float *out = p.out + ((int64_t)split * KT + k0) * 9 * CT + c0;
    float *red = lds2;                                    // [4 waves][32][32]
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave * 1024 + (8 * (v / 4) + 4 * h + v % 4) * 32 + r] = acc[tap][v];
        __syncthreads();
        for (int e = tid; e < 1024; e += 256)
            out[((e / 32) * 9 + tap) * CT + e % 32] = ((red[e] + red[1024 + e]) + red[2048 + e]) + red[3072 + e];
    }
}

struct WGradB2Cfg {
    bool use;
    int nsplit, per_split, bricks;
};

WGradB2Cfg wgrad2_brick_cfg(const ConvGeom &g)
{
    static const bool off = getenv("POOCH_NO_WGRAD2_BRICK") != nullptr;
    WGradB2Cfg c{false, 0, 0, 0};
    if (off || g.C % 32 != 0 || g.K % 32 != 0 || g.C > 256 || g.K > 256 || g.D != 1 || g.kd != 1 || g.kh != 3 || g.kw != 3) return c;
    if (g.sd != 1 || g.sh != 1 || g.sw != 1 || g.pd != 0 || g.ph != 1 || g.pw != 1) return c;
    if (g.Ho != g.H || g.Wo != g.W || g.N % 2 != 0 || g.H % C3_BH != 0 || g.W % C3_BW != 0) return c;
    // stand-alone, warmed up, against the generic kernels: 128 -> 128 at 56 x 56 124 against 118 TFLOP/s, at 24 x 24 124 against 117,
    // 64 -> 128 and 128 -> 64 124 against 84 and 81, 96 -> 96 121 against 69; 256 -> 256 124 against the eight-wave tile's 129
    if (g.K >= 256 && g.C >= 256) return c;
    c.bricks = (int)(g.rows_out() / (2 * C3_BH * C3_BW));
    const int nsub = (g.K / 32) * (g.C / 32);
    if (c.bricks < 4) return c;
    c.nsplit = 2 * NCU / nsub;                                       // as many workgroups as are resident at once,
    if (c.nsplit > c.bricks / 4) c.nsplit = c.bricks / 4;            // four bricks each at least
    if (c.nsplit < 1) c.nsplit = 1;
    c.per_split = (c.bricks + c.nsplit - 1) / c.nsplit;
    c.nsplit = (c.bricks + c.per_split - 1) / c.per_split;
    c.use = true;
    return c;
}

struct WHaloCfg {
    bool use;
    int gr, waves, P, PWpad, nseg_w, nseg, nsplit, seg_per_split, groups;
    int dy_blocks, row_blocks, lpw, buf_floats, nbuf;
    size_t lds_bytes;
};

constexpr size_t WGRAD_WS_CAP = (size_t)64 << 20;

// One way of running the halo kernel on a geometry: gr input rows per workgroup, `waves` wavefronts, an LDS budget per
// workgroup, so many workgroups in all.
// Segments: output rows cut into equal pieces of at most 64 pixels (a multiple of 8), as long as two buffers allow;
// then up to four buffers.  use stays false where the variant cannot serve the geometry.
WHaloCfg whalo_plan(const ConvGeom &g, int gr, int waves, size_t budget, int64_t workgroups)
{
    WHaloCfg c{};
    c.gr = gr;
    c.waves = waves;
    const int qc = g.C / 4;
    auto shape = [&](int P) {
        const int pw_units = ((P + 2) * qc + 63) / 64 * 64;      // a row's 16-byte pieces, in whole 64-lane blocks
        c.PWpad = pw_units / qc;
        c.row_blocks = pw_units / 64;
        c.dy_blocks = (P * g.K + 255) / 256;
        c.buf_floats = (c.dy_blocks + c.gr * c.row_blocks + 1) * 256;
        return (size_t)c.buf_floats * sizeof(float);
    };
    // the longest segment two buffers allow (each segment costs a barrier and a round of address arithmetic); then as
    // many buffers, up to four, as still fit
    int P = 0;
    for (int q = 64; q >= 8 && P == 0; q -= 8)
        if (2 * shape(q) <= budget) P = q;
    if (P == 0) return c;
    c.nseg_w = (g.Wo + P - 1) / P;
    c.P = ((g.Wo + c.nseg_w - 1) / c.nseg_w + 7) & ~7;           // pixels past the row's end carry a zero dy
    c.nbuf = (int)(budget / shape(c.P));
    c.nbuf = c.nbuf > 4 ? 4 : c.nbuf;
    c.lds_bytes = c.nbuf * shape(c.P);
    c.lpw = (c.dy_blocks + c.gr * c.row_blocks + c.waves - 1) / c.waves;
    if (c.lpw > WHALO_MAX_LPW) return c;
    while (c.nbuf > 2 && (c.nbuf - 2) * c.lpw > 8) --c.nbuf;   // (the counted wait knows 0 .. 8)
    const int64_t nseg = (int64_t)g.N * g.Do * g.Ho * c.nseg_w;
    if (nseg >= ((int64_t)1 << 30)) return c;
    c.nseg = (int)nseg;
    c.groups = g.kd * g.kh / c.gr;
    int64_t ns = workgroups / c.groups;
    const int64_t by_ws = (int64_t)(WGRAD_WS_CAP / ((size_t)g.K * g.taps() * g.C * sizeof(float)));
    if (ns > by_ws) ns = by_ws;
    if (ns > nseg) ns = nseg;
    if (ns < 1) ns = 1;
    c.seg_per_split = (int)((nseg + ns - 1) / ns);
    c.nsplit = (int)((nseg + c.seg_per_split - 1) / c.seg_per_split);
    // A workgroup's partial block is written once per workgroup: with very few segments each, that and the reduction
    // outweigh the gain (3 x 3 x 3 64 -> 64 at 32^3, three segments per workgroup: 72 TFLOP/s here against 75 generic;
    // from five on the kernels are level or this one ahead -- ResNet-50's 3 x 3 64 -> 64 at batch 16: 77 both, at batch 64: 96
    // against 79; 3 x 3 x 3 32 -> 32 at 64^3: 83 against 58).  Problems too small to matter either way (under 2 GFLOP) stay
    // here, so that small test shapes reach this kernel.
    if (c.seg_per_split < 4 && 2.0 * (double)g.rows_out() * g.K * (double)(g.taps() * g.C) > 2e9) return c;
    c.use = true;
    return c;
}

// whether the halo kernel serves this geometry, and how: unit strides, a 3-wide filter, 32 or 64 channels on
// both sides.  Rows per group: the three rows of one depth tap when a horizontal tap's accumulators fit 96 registers
// (32 -> 32, 32 -> 64, 64 -> 32 channels), else one.  Wavefronts: one per 32 x 32 block and horizontal tap -- nine for the three-row groups
// (two workgroups per compute unit, 76 KB of LDS each), twelve for 64 -> 64 (one workgroup per compute unit, up to 150 KB),
// three for a single filter row of 32 -> 32 (four per compute unit, 38 KB each).
// Workgroups: exactly as many as are resident at once, each walking its share of the segments from start to end.  More,
// smaller shares cost a ring fill, a partial block written and a ragged last round each; measured stand-alone, warmed up:
//   3 x 3 64 -> 64, 640 x 56 x 56 (twelve waves): 256 workgroups 105 TFLOP/s, 240: 99, 192: 80, 768: 105, 1536: 92
//   3 x 3 x 3 32 -> 32 at 192^3 (nine waves):     512 workgroups 94, 480: 89, 384: 71, 1024: 73, 3072: 82
//   3 x 3 x 3 64 -> 64 at 96^3 (twelve waves):    256 workgroups 98, 1536: 87
// (One wavefront per horizontal tap holding all four blocks of 64 -> 64 -- one LDS read per MFMA instead of two, three waves
// per workgroup, four workgroups per compute unit -- reached 99 on the last of these stand-alone and 74 inside a step, where
// the four workgroups per compute unit it depends on do not come together; it was taken out again.)
WHaloCfg whalo_cfg(const ConvGeom &g)
{
    static const bool off = getenv("POOCH_NO_HALO_WGRAD") != nullptr;
    if (off || g.sd != 1 || g.sh != 1 || g.sw != 1 || g.kw != 3) return WHaloCfg{};
    // 32 or 64 channels on either side; mixed widths (each wave holds the two blocks of its row and tap) only with three
    // filter rows per group.  (3 x 3 x 3 32 -> 64 at 96^3: 95 TFLOP/s against 80 with the generic kernel, 64 -> 32: 85 against 60.)
    if ((g.C != 32 && g.C != 64) || (g.K != 32 && g.K != 64)) return WHaloCfg{};
    if (g.K != g.C && g.kh != 3) return WHaloCfg{};
    WHaloCfg c;
    if (g.K != g.C) c = whalo_plan(g, 3, 9, 76 * 1024, 2 * NCU);
    else if (g.C == 32) c = g.kh == 3 ? whalo_plan(g, 3, 9, 76 * 1024, 2 * NCU) : whalo_plan(g, 1, 3, 38 * 1024, 4 * NCU);
    else c = whalo_plan(g, 1, 12, 150 * 1024, NCU);
    return c.use ? c : WHaloCfg{};
}

template <int KB, int CB, int GR, int GW, int IW, int JW>
hipError_t launch_whalo(WHaloP p, const WHaloCfg &c, hipStream_t s)
{
    constexpr int NWV = 3 * (GR / GW) * (KB / IW) * (CB / JW);
    if (c.waves != NWV || c.lpw > WHALO_MAX_LPW) return hipErrorInvalidValue;
    p.total = p.nsplit * p.groups;
    p.chunk = (p.total + NXCD - 1) / NXCD;
    if (c.lds_bytes > 64 * 1024) {   // more dynamic LDS than the default limit: raised once per kernel (no allocation)
        static bool raised = false;
        if (!raised) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_halo_kernel<KB, CB, GR, GW, IW, JW>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    wgrad_halo_kernel<KB, CB, GR, GW, IW, JW><<<dim3(p.chunk * NXCD), dim3(64 * NWV), c.lds_bytes, s>>>(p);
    return hipGetLastError();
}

hipError_t dispatch_whalo(const WHaloP &hp, const WHaloCfg &hc, hipStream_t s)
{
    if (hp.K == 64 && hp.C == 32) return hc.gr == 3 ? launch_whalo<2, 1, 3, 1, 2, 1>(hp, hc, s) : hipErrorInvalidValue;
    if (hp.K == 32 && hp.C == 64) return hc.gr == 3 ? launch_whalo<1, 2, 3, 1, 1, 2>(hp, hc, s) : hipErrorInvalidValue;
    if (hp.K != hp.C) return hipErrorInvalidValue;
    if (hp.K == 32) return hc.gr == 3 ? launch_whalo<1, 1, 3, 1, 1, 1>(hp, hc, s) : launch_whalo<1, 1, 1, 1, 1, 1>(hp, hc, s);
    return hc.gr == 1 ? launch_whalo<2, 2, 1, 1, 1, 1>(hp, hc, s) : hipErrorInvalidValue;
}

struct WGradCfg {
    int bm, bn, nsplit, chunk_rows;
    int big;   // 0: the bm x bn tile with four waves; 1: 256 x 128 with eight; 2: 128 x 256 with eight
};

WGradCfg wgrad_cfg(const ConvGeom &g)
{
    WGradCfg c;
    const int64_t M = g.rows_out(), Kred = g.taps() * g.C;
    c.bm = g.K <= 32 ? 32 : (g.K <= 64 ? 64 : 128);
    // column tiles: 128 wide; 64 when that already covers the row, and for few output channels under
    // several 16-channel-aligned taps.  Measured on the 64-output-channel ResNet-50 layers at batch 640:
    // 1x1 256->64 0.62 ms at 128 (four waves of 32 x 64) against 0.70 ms at 64; 3x3 64->64 1.90 ms at 64
    // against 1.96 ms at 128; the 4-channel stem 2.5 ms with four waves of 32 x 64 against 3.5 ms with two of 64 x 64
    // (up to 32 output channels: 3x3x3 32->32 at 192^3 6.8 ms at 128 against 7.7 ms at 64)
    c.bn = (Kred <= 64 || (c.bm == 64 && g.C % 16 == 0 && g.taps() > 1)) ? 64 : 128;
    const int64_t tiles = ((g.K + c.bm - 1) / c.bm) * ((Kred + c.bn - 1) / c.bn);
    // about as many workgroups as are resident at once (four per compute unit; measured on ResNet-50's layers at batch 640:
    // a target of 512 or 768 loses up to 45 %, 1536 and 2048 are level with 1024), but each split keeps at
    // least 256 rows so that its epilogue (a full tile written to the workspace) stays small
    int64_t ns = (1024 + tiles - 1) / tiles;
    const int64_t max_by_rows = (M + 255) / 256;
    if (ns > max_by_rows) ns = max_by_rows;
    const int64_t max_by_ws = (int64_t)(WGRAD_WS_CAP / ((size_t)g.K * Kred * sizeof(float)));
    if (ns > max_by_ws) ns = max_by_ws;
    if (ns < 1) ns = 1;
    int64_t chunk = (M + ns - 1) / ns;
    chunk = (chunk + BK - 1) / BK * BK;
    c.chunk_rows = (int)chunk;
    c.nsplit = (int)((M + chunk - 1) / chunk);
    // Eight waves on a double tile where the output has room for it (the split count stays the one
    // of the 128 x 128 tiling: half as many workgroups of twice the size).  Measured at batch 640:
    // 256 x 128 on 256 or more output channels 126 - 130 TFLOP/s against 117 - 119; 128 x 256 on 1x1
    // filters into 128 channels 0.535 against 0.571 ms -- but 1.77 against 1.25 ms under 3x3 taps, hence not there
    c.big = 0;
    if (c.bm == 128 && c.bn == 128) {
        if (g.K >= 256) c.big = 1;
        else if (Kred >= 256 && g.taps() == 1) c.big = 2;
    }
    return c;
}

template <int WGM, int WGN, int TM, int TN>
hipError_t launch_wgrad(WGradP p, bool veca, bool vecb, hipStream_t s)
{
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    const int tiles_m = (p.K + BM - 1) / BM;
    p.tiles_n = (p.Kred + BN - 1) / BN;
    p.tiles = tiles_m * p.tiles_n;
    p.total = p.tiles * p.nsplit;
    p.chunk = (p.total + NXCD - 1) / NXCD;
    const dim3 grid(p.chunk * NXCD), block(64 * WGM * WGN);
    if (veca && vecb) wgrad_kernel<WGM, WGN, TM, TN, true, true><<<grid, block, 0, s>>>(p);
    else if (veca) wgrad_kernel<WGM, WGN, TM, TN, true, false><<<grid, block, 0, s>>>(p);
    else if (vecb) wgrad_kernel<WGM, WGN, TM, TN, false, true><<<grid, block, 0, s>>>(p);
    else wgrad_kernel<WGM, WGN, TM, TN, false, false><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
}

}  // namespace

namespace {
IGemmP fwd_params(const float *x, const float *w_krsc, float *y, const ConvGeom &g)
{
    IGemmP p;
    p.src = x; p.wgt = w_krsc; p.dst = y; p.stats = nullptr;
    p.M = (int)g.rows_out(); p.Nout = g.K; p.Kred = (int)(g.taps() * g.C); p.Cs = g.C;
    p.Dr = g.Do; p.Hr = g.Ho; p.Wr = g.Wo; p.Ds = g.D; p.Hs = g.H; p.Ws = g.W;
    p.kd = g.kd; p.kh = g.kh; p.kw = g.kw; p.sd = g.sd; p.sh = g.sh; p.sw = g.sw; p.pd = g.pd; p.ph = g.ph; p.pw = g.pw;
    p.dst_strided = 0; p.DD = p.HD = p.WD = p.SD = p.SH = p.SW = 0;
    p.live = g.Clive;
    return p;
}

// the data gradient as a GEMM over the INPUT positions (not the scatter form of a strided 1 x 1 filter)
IGemmP dgrad_params(const float *dy, const float *w_crsk, float *dx, const ConvGeom &g)
{
    IGemmP p;
    p.src = dy; p.wgt = w_crsk; p.dst = dx; p.stats = nullptr; p.live = 0;
    p.M = (int)g.rows_in(); p.Nout = g.C; p.Kred = (int)(g.taps() * g.K); p.Cs = g.K;
    p.Dr = g.D; p.Hr = g.H; p.Wr = g.W; p.Ds = g.Do; p.Hs = g.Ho; p.Ws = g.Wo;
    p.kd = g.kd; p.kh = g.kh; p.kw = g.kw; p.sd = g.sd; p.sh = g.sh; p.sw = g.sw; p.pd = g.pd; p.ph = g.ph; p.pw = g.pw;
    p.dst_strided = 0; p.DD = p.HD = p.WD = p.SD = p.SH = p.SW = 0;
    return p;
}
}  // namespace

bool conv_fwd_bn_tiles(const float *x, const float *w_krsc, const ConvGeom &g, int *tiles_m, int *rows_per_tile)
{
    if (!geom_ok(g) || !tiles_m || !rows_per_tile || g.K % 4 != 0) return false;
    const IGemmP p = fwd_params(x, w_krsc, nullptr, g);
    const bool vec = (p.Cs % 4 == 0) && ((uintptr_t)p.src % 16 == 0) && ((uintptr_t)p.wgt % 16 == 0);
    if (!vec || igemm_linear_mode(p.Cs, false, true, false) == 0) return false;
    int lay[2] = {0, 0};
    if (dispatch_igemm<false>(p, false, nullptr, lay) != hipSuccess) return false;
    *tiles_m = lay[0];
    *rows_per_tile = lay[1];
    return true;
}

size_t conv_fwd_workspace(const ConvGeom &g)
{
    if (!geom_ok(g)) return 0;
    const int lin = g.C % 4 == 0 ? igemm_linear_mode(g.C, false, true, false) : 0;
    const SplitK sk = igemm_splitk((int)g.rows_out(), g.K, (int)(g.taps() * g.C), lin, false);
    return sk.ksplit > 1 ? (size_t)sk.ksplit * g.rows_out() * g.K * sizeof(float) : 0;
}

hipError_t conv_fwd(const float *x, const float *w_krsc, float *y, const ConvGeom &g, hipStream_t s, float *bn_tiles, float *workspace)
{
    if (!x || !w_krsc || !y || !geom_ok(g)) return hipErrorInvalidValue;
    IGemmP p = fwd_params(x, w_krsc, y, g);
    if (bn_tiles) {
        int tm, rows;
        if ((uintptr_t)bn_tiles % 16 != 0 || !conv_fwd_bn_tiles(x, w_krsc, g, &tm, &rows)) return hipErrorInvalidValue;
        p.stats = bn_tiles;
    }
    return dispatch_igemm<false>(p, false, s, nullptr, workspace);
}

// a strided 1x1 filter without padding touches only every (sd,sh,sw)-th input position: its
// data gradient is a plain GEMM over the OUTPUT rows scattered to those positions; all other
// positions receive zero
bool pointwise_strided(const ConvGeom &g)
{
    return g.taps() == 1 && g.pd == 0 && g.ph == 0 && g.pw == 0 && (g.sd > 1 || g.sh > 1 || g.sw > 1);
}

size_t conv_dgrad_workspace(const ConvGeom &g)
{
    if (!geom_ok(g) || pointwise_strided(g)) return 0;
    const int lin = g.K % 4 == 0 ? igemm_linear_mode(g.K, true, g.sd == 1 && g.sh == 1 && g.sw == 1, false) : 0;
    const SplitK sk = igemm_splitk((int)g.rows_in(), g.C, (int)(g.taps() * g.K), lin, false);
    return sk.ksplit > 1 ? (size_t)sk.ksplit * g.rows_in() * g.C * sizeof(float) : 0;
}

hipError_t conv_dgrad(const float *dy, const float *w_crsk, float *dx, const ConvGeom &g, bool accumulate, hipStream_t s, float *workspace)
{
    if (!dy || !w_crsk || !dx || !geom_ok(g)) return hipErrorInvalidValue;
    IGemmP p;
    p.stats = nullptr;
    p.live = 0;
    if (pointwise_strided(g)) {
        if (!accumulate) {
            const hipError_t e = fill_zero(dx, g.rows_in() * g.C, s);
            if (e != hipSuccess) return e;
        }
        p.src = dy; p.wgt = w_crsk; p.dst = dx;
        p.M = (int)g.rows_out(); p.Nout = g.C; p.Kred = g.K; p.Cs = g.K;
        p.Dr = g.Do; p.Hr = g.Ho; p.Wr = g.Wo; p.Ds = g.Do; p.Hs = g.Ho; p.Ws = g.Wo;
        p.kd = p.kh = p.kw = 1; p.sd = p.sh = p.sw = 1; p.pd = p.ph = p.pw = 0;
        p.dst_strided = 1; p.DD = g.D; p.HD = g.H; p.WD = g.W; p.SD = g.sd; p.SH = g.sh; p.SW = g.sw;
        // rows that are not written keep their zeros; the scattered rows are stored over them, or added to what is there
        return dispatch_igemm<false>(p, accumulate, s);
    }
    p = dgrad_params(dy, w_crsk, dx, g);
    return dispatch_igemm<true>(p, accumulate, s, nullptr, workspace);
}

namespace {
// tag of the igemm instantiation dispatch_igemm() picks: tile shape, load path, direction.  one_tap: a single filter tap
// and no padding (the plain-GEMM path where whole slices per tap apply)
const char *igemm_tag(int64_t rows, int nout, int cs, bool unit_stride, bool dgrad, int kred, bool one_tap)
{
    const bool vec = cs % 4 == 0;
    const int lin = vec ? igemm_linear_mode(cs, dgrad, unit_stride, false) : 0;
    static const bool no_gemm = getenv("POOCH_NO_GEMM_PATH") != nullptr, narrow = getenv("POOCH_NO_WIDE_SLICE") != nullptr;
    const bool gemm = lin == 1 && one_tap && !no_gemm;
    std::string name = "igemm_kernel<";
    if (vec && igemm_splitk((int)rows, nout, kred, lin, false).ksplit > 1) {
        name += "2,2,2,2,";
    } else if (nout > 64 && ((rows + 127) / 128) * ((nout + 127) / 128) < 640) {
        name += "2,2,1,1,";
    } else {
        name += nout <= 32 ? "4,1,2,1," : (nout <= 64 ? "4,1,2,2," : "2,2,2,2,");
    }
    const bool split = vec && igemm_splitk((int)rows, nout, kred, lin, false).ksplit > 1;
    const bool wide = !split && nout <= 32 && lin == 1 && !gemm && cs % 32 == 0 && !narrow &&
                      !(nout > 64 && ((rows + 127) / 128) * ((nout + 127) / 128) < 640);
    name += !vec ? "scalar" : (lin == 2 ? "vec+tap" : (gemm ? "vec+gemm" : (lin == 1 ? (wide ? "vec+lin32" : "vec+lin") : "vec")));
    name += dgrad ? ",dgrad" : ",fwd";
    if (split) name += ",splitk";
    name += ">";
    static std::map<std::string, std::string> names;   // (the caller keeps the pointer)
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    return names.emplace(name, name).first->second.c_str();
}
}  // namespace

const char *conv_fwd_kernel(const ConvGeom &g, bool bn_tiles)
{
    if (conv3_halo_ok(fwd_params(nullptr, nullptr, nullptr, g), true)) return bn_tiles ? "conv3_halo_kernel<fwd+bnstats>" : "conv3_halo_kernel<fwd>";
    if (conv3_c1_ok(fwd_params(nullptr, nullptr, nullptr, g))) return bn_tiles ? "conv3_c1_kernel<fwd+bnstats>" : "conv3_c1_kernel<fwd>";
    if (stem7_ok(fwd_params(nullptr, nullptr, nullptr, g))) return bn_tiles ? "stem7_fwd_kernel<fwd+bnstats>" : "stem7_fwd_kernel<fwd>";
    const bool one_tap = g.taps() == 1 && g.pd == 0 && g.ph == 0 && g.pw == 0;
    const char *plain = igemm_tag(g.rows_out(), g.K, g.C, true, false, (int)(g.taps() * g.C), one_tap);
    if (!bn_tiles) return plain;
    // the variant that also leaves batch-normalisation statistics is a kernel of its own
    static std::map<std::string, std::string> names;
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    std::string &v = names[plain];
    if (v.empty()) {
        v = plain;
        v.insert(v.size() - 1, "+bnstats");
    }
    return v.c_str();
}

const char *conv_dgrad_kernel(const ConvGeom &g)
{
    if (pointwise_strided(g)) return igemm_tag(g.rows_out(), g.C, g.K, true, false, 0, true);   // scatter GEMM over the output rows (never split)
    if (conv3_halo_ok(dgrad_params(nullptr, nullptr, nullptr, g), true)) return "conv3_halo_kernel<dgrad>";
    const bool one_tap = g.taps() == 1 && g.pd == 0 && g.ph == 0 && g.pw == 0;
    return igemm_tag(g.rows_in(), g.C, g.K, g.sd == 1 && g.sh == 1 && g.sw == 1, true, (int)(g.taps() * g.K), one_tap);
}

const char *conv_wgrad_kernel(const ConvGeom &g)
{
    if (geom_ok(g)) {
        if (wgrad3_c1_cfg(g).use) return "wgrad3_c1_kernel";
        if (stem7_wgrad_cfg(g).use) return "stem7_wgrad_kernel";
        if (wgrad3_brick_cfg(g).use) return "wgrad3_brick_kernel";
        if (wgrad2_brick_cfg(g).use) return "wgrad2_brick_kernel";
        const WHaloCfg hc = whalo_cfg(g);
        if (hc.use) {
            if (g.K != g.C) return g.K == 64 ? "wgrad_halo_kernel<2,1,3>" : "wgrad_halo_kernel<1,2,3>";
            return g.K == 32 ? (hc.gr == 3 ? "wgrad_halo_kernel<1,1,3>" : "wgrad_halo_kernel<1,1,1>") : "wgrad_halo_kernel<2,2,1>";
        }
    }
    const WGradCfg c = wgrad_cfg(g);
    if (c.bn == 64) return c.bm == 32 ? "wgrad_kernel<1,2,1,1>" : (c.bm == 64 ? "wgrad_kernel<2,2,1,1>" : "wgrad_kernel<2,2,2,1>");
    if (c.big) return c.big == 1 ? "wgrad_kernel<4,2,2,2>" : "wgrad_kernel<2,4,2,2>";
    return c.bm == 32 ? "wgrad_kernel<1,2,1,2>" : (c.bm == 64 ? "wgrad_kernel<2,2,1,2>" : "wgrad_kernel<2,2,2,2>");
}

size_t conv_wgrad_workspace(const ConvGeom &g)
{
    if (!geom_ok(g)) return 0;
    const WGradC1Cfg c1 = wgrad3_c1_cfg(g);
    if (c1.use) return (size_t)c1.nsplit * g.K * g.taps() * g.C * sizeof(float);
    const WGradB3Cfg b3 = wgrad3_brick_cfg(g);
    if (b3.use) return (size_t)b3.nsplit * g.K * g.taps() * g.C * sizeof(float);
    const Stem7WCfg s7 = stem7_wgrad_cfg(g);
    if (s7.use) return (size_t)s7.nsplit * g.K * g.taps() * g.C * sizeof(float);
    const WGradB2Cfg b2 = wgrad2_brick_cfg(g);
    if (b2.use) return (size_t)b2.nsplit * g.K * g.taps() * g.C * sizeof(float);
    const WHaloCfg hc = whalo_cfg(g);
    if (hc.use) return (size_t)hc.nsplit * g.K * g.taps() * g.C * sizeof(float);
    const WGradCfg c = wgrad_cfg(g);
    return c.nsplit > 1 ? (size_t)c.nsplit * g.K * g.taps() * g.C * sizeof(float) : 0;
}

hipError_t conv_wgrad(const float *dy, const float *x, float *dw_krsc, float *workspace, const ConvGeom &g, hipStream_t s)
{
    if (!dy || !x || !dw_krsc || !geom_ok(g)) return hipErrorInvalidValue;
    const WGradC1Cfg c1 = wgrad3_c1_cfg(g);
    if (c1.use) {
        if (!workspace) return hipErrorInvalidValue;
        WGradC1P cp;
        cp.dy = dy; cp.x = x; cp.out = workspace;
        cp.N = g.N; cp.D = g.D; cp.H = g.H; cp.W = g.W; cp.Cs = g.C;
        cp.bricks = c1.bricks; cp.per_wave = c1.per_wave;
        wgrad3_c1_kernel<<<dim3(c1.nsplit), dim3(512), 0, s>>>(cp);
        const hipError_t ce = hipGetLastError();
        if (ce != hipSuccess) return ce;
        const int64_t nel = (int64_t)g.K * g.taps() * g.C;
        reduce_splits_kernel<<<dim3((unsigned)((nel + 63) / 64)), dim3(256), 0, s>>>(workspace, dw_krsc, nel, c1.nsplit);
        return hipGetLastError();
    }
    const Stem7WCfg s7 = stem7_wgrad_cfg(g);
    if (s7.use) {
        if (!workspace || (uintptr_t)x % 16 != 0) return hipErrorInvalidValue;
        Stem7WP sp;
        sp.dy = dy; sp.x = x; sp.out = workspace;
        sp.N = g.N; sp.H = g.H; sp.W = g.W; sp.Ho = g.Ho; sp.Wo = g.Wo;
        sp.tiles = s7.tiles; sp.per_wg = s7.per_wg;
        stem7_wgrad_kernel<<<dim3(s7.nsplit), dim3(256), 0, s>>>(sp);
        const hipError_t se = hipGetLastError();
        if (se != hipSuccess) return se;
        const int64_t nel = (int64_t)g.K * g.taps() * g.C;
        reduce_splits_kernel<<<dim3((unsigned)((nel + 63) / 64)), dim3(256), 0, s>>>(workspace, dw_krsc, nel, s7.nsplit);
        return hipGetLastError();
    }
    const WGradB3Cfg b3 = wgrad3_brick_cfg(g);
    if (b3.use) {
        if (!workspace || (uintptr_t)dy % 16 != 0 || (uintptr_t)x % 16 != 0) return hipErrorInvalidValue;
        WGradB3P bp;
        bp.dy = dy; bp.x = x; bp.out = workspace;
        bp.N = g.N; bp.D = g.D; bp.H = g.H; bp.W = g.W; bp.K = g.K; bp.C = g.C;
        bp.bricks = b3.bricks; bp.per_split = b3.per_split;
        static bool raised = false;     // more dynamic LDS than the default limit: raised once (no allocation)
        if (!raised) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad3_brick_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
        wgrad3_brick_kernel<<<dim3(b3.nsplit * (g.K / 32) * (g.C / 32)), dim3(256), WGRAD3_BRICK_LDS, s>>>(bp);
        const hipError_t be = hipGetLastError();
        if (be != hipSuccess) return be;
        const int64_t nel = (int64_t)g.K * g.taps() * g.C;
        reduce_splits_kernel<<<dim3((unsigned)((nel + 63) / 64)), dim3(256), 0, s>>>(workspace, dw_krsc, nel, b3.nsplit);
        return hipGetLastError();
    }
    const WGradB2Cfg b2 = wgrad2_brick_cfg(g);
    if (b2.use) {
        if (!workspace || (uintptr_t)dy % 16 != 0 || (uintptr_t)x % 16 != 0) return hipErrorInvalidValue;
        WGradB2P bp;
        bp.dy = dy; bp.x = x; bp.out = workspace;
        bp.N = g.N; bp.H = g.H; bp.W = g.W; bp.K = g.K; bp.C = g.C;
        bp.bricks = b2.bricks; bp.per_split = b2.per_split;
        wgrad2_brick_kernel<<<dim3(b2.nsplit * (g.K / 32) * (g.C / 32)), dim3(256), 0, s>>>(bp);
        const hipError_t be = hipGetLastError();
        if (be != hipSuccess) return be;
        const int64_t nel = (int64_t)g.K * g.taps() * g.C;
        reduce_splits_kernel<<<dim3((unsigned)((nel + 63) / 64)), dim3(256), 0, s>>>(workspace, dw_krsc, nel, b2.nsplit);
        return hipGetLastError();
    }
    const WHaloCfg hc = whalo_cfg(g);
    if (hc.use) {
        // (the workspace is sized for this path: no falling back to the generic kernel's split count)
        if (!workspace || (uintptr_t)dy % 16 != 0 || (uintptr_t)x % 16 != 0 || (uintptr_t)workspace % 16 != 0) return hipErrorInvalidValue;
        WHaloP hp;
        hp.dy = dy; hp.x = x; hp.out = workspace;
        hp.K = g.K; hp.C = g.C; hp.Kred = (int)(g.taps() * g.C);
        hp.N = g.N; hp.D = g.D; hp.H = g.H; hp.W = g.W; hp.Do = g.Do; hp.Ho = g.Ho; hp.Wo = g.Wo;
        hp.kd = g.kd; hp.kh = g.kh; hp.pd = g.pd; hp.ph = g.ph; hp.pw = g.pw;
        hp.P = hc.P; hp.PW = hc.P + 2; hp.PWpad = hc.PWpad; hp.nseg_w = hc.nseg_w; hp.nseg = hc.nseg;
        hp.dy_blocks = hc.dy_blocks; hp.row_blocks = hc.row_blocks; hp.lpw = hc.lpw; hp.buf_floats = hc.buf_floats; hp.nbuf = hc.nbuf;
        hp.seg_per_split = hc.seg_per_split; hp.nsplit = hc.nsplit; hp.groups = hc.groups;
        const hipError_t he = dispatch_whalo(hp, hc, s);
        if (he != hipSuccess) return he;
        const int64_t nel = (int64_t)g.K * hp.Kred;
        reduce_splits_kernel<<<dim3((unsigned)((nel + 63) / 64)), dim3(256), 0, s>>>(workspace, dw_krsc, nel, hc.nsplit);
        return hipGetLastError();
    }
    const WGradCfg c = wgrad_cfg(g);
    if (c.nsplit > 1 && !workspace) return hipErrorInvalidValue;
    WGradP p;
    p.dy = dy; p.x = x; p.out = c.nsplit > 1 ? workspace : dw_krsc;
    p.M = (int)g.rows_out(); p.K = g.K; p.Kred = (int)(g.taps() * g.C); p.C = g.C;
    p.Do = g.Do; p.Ho = g.Ho; p.Wo = g.Wo; p.D = g.D; p.H = g.H; p.W = g.W;
    p.kd = g.kd; p.kh = g.kh; p.kw = g.kw; p.sd = g.sd; p.sh = g.sh; p.sw = g.sw; p.pd = g.pd; p.ph = g.ph; p.pw = g.pw;
    p.chunk_rows = c.chunk_rows; p.nsplit = c.nsplit; p.tiles_n = 0;
    const bool veca = (g.K % 4 == 0) && ((uintptr_t)dy % 16 == 0);
    const bool vecb = (g.C % 4 == 0) && ((uintptr_t)x % 16 == 0);
    hipError_t e;
    if (c.bn == 64) {
        if (c.bm == 32) e = launch_wgrad<1, 2, 1, 1>(p, veca, vecb, s);
        else if (c.bm == 64) e = launch_wgrad<2, 2, 1, 1>(p, veca, vecb, s);
        else e = launch_wgrad<2, 2, 2, 1>(p, veca, vecb, s);
    } else {
        if (c.bm == 32) e = launch_wgrad<1, 2, 1, 2>(p, veca, vecb, s);
        else if (c.bm == 64) e = launch_wgrad<2, 2, 1, 2>(p, veca, vecb, s);
        else if (c.big == 1) e = launch_wgrad<4, 2, 2, 2>(p, veca, vecb, s);
        else if (c.big == 2) e = launch_wgrad<2, 4, 2, 2>(p, veca, vecb, s);
        else e = launch_wgrad<2, 2, 2, 2>(p, veca, vecb, s);
    }
    if (e != hipSuccess) return e;
    if (c.nsplit > 1) {
        const int64_t n = (int64_t)g.K * p.Kred;
        reduce_splits_kernel<<<dim3((unsigned)((n + 63) / 64)), dim3(256), 0, s>>>(workspace, dw_krsc, n, c.nsplit);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace pk
