// C ABI of the out-of-core training step: context, layer graph, resident-region layout,
// parameter / batch marshalling, the command-list executor with its swap engine (paper
// section 3.1) and recompute executor (section 3.2), the runtime profiler (section 4.2)
// and the entry points of the classification (section 4.4).
//
// Execution model: a plan is a static command list (plan.cpp).  pooch_step() replays it on
// three caller-owned HIP streams -- compute, device-to-host, host-to-device -- with every
// cross-stream dependency expressed as an event record / wait pair, so the host enqueues a
// whole step without blocking and synchronises once at the end.
#include "../../include/pooch.h"
#include "core.hpp"
#include "kernels.h"

#include <algorithm>
#include <array>
#include <cstdlib>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>

using namespace pooch;

// ---- static scratch of pooch_step_static_scratch ------------------------------------------------------------
// Device memory the kernels of a step use beyond their inputs and outputs -- the filter gradients' split-K
// partials, the batch normalisations' reduction partials and per-tile statistics, the per-sample losses -- for
// callers that may not allocate: a file-scope array instead of a range of the arena.  Every GPU the library runs
// on holds its own copy from the moment the code object is loaded there until the process ends.  In host code the
// array's name is only a handle: its device address comes from hipGetSymbolAddress, once per device
// (static_scratch_for), and that address is what kernels and copies are given.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)128 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};   // per device: address of that device's copy of `scratch`

// address of `scratch` on `device`; looked up on first use with that device current
hipError_t static_scratch_for(int device, void **out)
{
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        int current = -1;
        hipError_t e = hipGetDevice(&current);
        if (e != hipSuccess) return e;
        if (current != device) {
            e = hipSetDevice(device);
            if (e != hipSuccess) return e;
        }
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (current != device) (void)hipSetDevice(current);
        if (e != hipSuccess) return e;
        if (!ptr || (uintptr_t)ptr % 256 != 0) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}
}  // namespace

namespace {

struct ParamInfo {
    int node;
    int which;            // 0: filter / gamma / fc weight, 1: beta / fc bias
    int64_t numel;        // logical element count (what the caller passes in and gets back)
    int64_t dev_numel;    // elements on the device (larger when the input channels are padded)
    int64_t off_val;      // resident offsets (bytes from the arena base)
    int64_t off_val_t;    // transposed filter copy for the data gradient, or -1
    int64_t off_grad;
};

struct Timing {
    std::vector<int> start, stop;      // per command: indices into the timing-event pool, -1 = untimed
    std::vector<char> own_start;       // the start event is this command's own (else: the stop event of the command before it on its stream)
    std::vector<int> rstart, rstop;    // profile mode: the re-forward run right after a forward
    std::vector<int> mid;              // conv / fc backward: between the filter and the data gradient
};

}  // namespace

struct pooch_ctx {
    char *arena = nullptr;
    size_t arena_bytes = 0;
    char *pinned = nullptr;
    size_t pinned_bytes = 0;
    hipStream_t st[3] = {nullptr, nullptr, nullptr};

    Graph G;
    bool finalized = false;
    std::vector<ParamInfo> params;
    std::vector<int64_t> off_mean, off_istd;  // per node (BN only), resident offsets
    std::vector<int64_t> off_rmean, off_rvar; // running averages of the same layers
    std::vector<int64_t> off_mask;            // per node: resident offset of its one-bit ReLU mask, -1 where it keeps none
    float bn_decay = 0.9f;
    // what a step needs before it may touch the device: a batch (the labels index the logits) and every parameter;
    // and what an update or a read-back of gradients needs: a step that has run
    bool has_batch = false, has_grads = false;
    std::vector<char> param_set;
    int64_t off_input = 0, off_labels = 0, off_ws_wgrad = 0, off_ws_bn = 0, off_loss_ps = 0, off_loss = 0;
    int64_t ws_wgrad_bytes = 0, ws_bn_bytes = 0, loss_ps_bytes = 0;   // sizes of the three scratch ranges (256-byte rounded)
    char *static_scratch = nullptr;         // this context's GPU's copy of the static scratch array (compute contexts)
    int64_t resident_bytes = 0;
    int nclasses = 0;
    // device channel count of the network input: a 3-channel input read only by convolutions is
    // stored with a zero fourth channel (and those filters with a zero fourth input channel), so
    // that its rows are 16-byte vectors like every other tensor's
    int in_cdev = 0;
    // A convolution whose result goes straight into a batch normalisation leaves that layer's
    // statistics per row tile while it writes (stats_to[conv] = the BN node, stats_from[bn] = the
    // conv node, stats_tiles[bn] = {row tiles, rows per tile}); -1 where the BN reads its input itself.
    std::vector<int> stats_to, stats_from;
    std::vector<std::array<int, 2>> stats_tiles;

    Profile prof;
    bool has_plan = false;
    bool profile_newer_than_plan = false;   // the profile changed while a plan was installed (see pooch_plan)
    std::vector<uint8_t> cls;
    bool ahead = true;
    Schedule sched;
    double predicted_ms = 0.0;
    int64_t evals = 0;
    int restarts = 8;
    double last_step_ms = 0.0;
    // samples gathered by pooch_profile_step, turned into a profile by pooch_finish_profile
    std::vector<std::vector<double>> smp_f, smp_b, smp_r, smp_o, smp_i;
    Schedule prof_sched;
    bool prof_sched_ok = false;

    std::vector<hipEvent_t> sync_events;    // no timing
    std::vector<hipEvent_t> timing_events;  // with timing
    std::vector<float *> capture;           // per node host destination or nullptr
    std::vector<float> host_tmp;
    int64_t fail_at = -1;                   // test aid (pooch_inject_failure): command of the next replay that fails
    std::string err;
};

namespace {

int64_t round_up(int64_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }

pooch_status fail(pooch_ctx *c, pooch_status s, const std::string &msg)
{
    if (c) c->err = msg;
    return s;
}

#define HIPCHK(expr)                                                                                       \
    do {                                                                                                   \
        hipError_t e_ = (expr);                                                                            \
        if (e_ != hipSuccess) return fail(c, POOCH_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

pk::ConvGeom conv_geom(const Graph &G, int i, int in_cdev)
{
    const Node &nd = G.nodes[i];
    const Node &x = G.nodes[nd.in[0]];
    pk::ConvGeom g;
    g.N = (int)x.N; g.C = nd.in[0] == 0 ? in_cdev : (int)x.C; g.D = (int)x.sp[0]; g.H = (int)x.sp[1]; g.W = (int)x.sp[2];
    g.Clive = nd.in[0] == 0 && in_cdev != (int)x.C ? (int)x.C : 0;
    g.K = (int)nd.C;
    g.Do = (int)nd.sp[0]; g.Ho = (int)nd.sp[1]; g.Wo = (int)nd.sp[2];
    if (nd.op == OP_FC) {
        // a fully-connected layer is a convolution whose filter covers the whole input
        g.kd = g.D; g.kh = g.H; g.kw = g.W; g.sd = g.sh = g.sw = 1; g.pd = g.ph = g.pw = 0;
    } else {
        g.kd = nd.k[0]; g.kh = nd.k[1]; g.kw = nd.k[2];
        g.sd = nd.st[0]; g.sh = nd.st[1]; g.sw = nd.st[2];
        g.pd = nd.pd[0]; g.ph = nd.pd[1]; g.pw = nd.pd[2];
    }
    return g;
}

pk::PoolGeom pool_geom(const Graph &G, int i)
{
    const Node &nd = G.nodes[i];
    const Node &x = G.nodes[nd.in[0]];
    pk::PoolGeom g;
    g.N = (int)x.N; g.C = (int)x.C; g.D = (int)x.sp[0]; g.H = (int)x.sp[1]; g.W = (int)x.sp[2];
    g.Do = (int)nd.sp[0]; g.Ho = (int)nd.sp[1]; g.Wo = (int)nd.sp[2];
    g.kd = nd.k[0]; g.kh = nd.k[1]; g.kw = nd.k[2];
    g.sd = nd.st[0]; g.sh = nd.st[1]; g.sw = nd.st[2];
    g.pd = nd.pd[0]; g.ph = nd.pd[1]; g.pw = nd.pd[2];
    return g;
}

// logical K,C,taps  <->  device K,taps,Cd and Cd,taps,K (Cd >= C; device buffers pre-zeroed by the caller)
void filter_to_device_layouts(const float *kcr, int64_t K, int64_t C, int64_t Cd, int64_t T, float *krc, float *crk)
{
    for (int64_t k = 0; k < K; ++k)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t t = 0; t < T; ++t) {
                const float v = kcr[(k * C + c) * T + t];
                krc[(k * T + t) * Cd + c] = v;
                crk[(c * T + t) * K + k] = v;
            }
}

void filter_from_device_layout(const float *krc, int64_t K, int64_t C, int64_t Cd, int64_t T, float *kcr)
{
    for (int64_t k = 0; k < K; ++k)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t t = 0; t < T; ++t) kcr[(k * C + c) * T + t] = krc[(k * T + t) * Cd + c];
}

// logical N,C,S <-> device N,S,Cd (Cd >= C; device buffer pre-zeroed by the caller)
void act_to_device_layout(const float *ncs, int64_t N, int64_t C, int64_t Cd, int64_t S, float *nsc)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c) {
            const float *src = ncs + (n * C + c) * S;
            float *dst = nsc + n * S * Cd + c;
            for (int64_t s = 0; s < S; ++s) dst[s * Cd] = src[s];
        }
}

void act_from_device_layout(const float *nsc, int64_t N, int64_t C, int64_t S, float *ncs)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c) {
            float *dst = ncs + (n * C + c) * S;
            const float *src = nsc + n * S * C + c;
            for (int64_t s = 0; s < S; ++s) dst[s] = src[s * C];
        }
}

struct Exec {
    pooch_ctx *c;
    const Schedule &S;
    hipEvent_t mid = nullptr;  // when set, recorded between the filter gradient and the data gradient
    // kernel scratch: ranges of the arena's resident region, or of the static scratch array
    float *ws_wgrad, *ws_bn, *loss_ps;
    Exec(pooch_ctx *ctx, const Schedule &s, bool static_scratch) : c(ctx), S(s)
    {
        char *base = static_scratch ? ctx->static_scratch : ctx->arena + ctx->off_ws_wgrad;
        // the three ranges lie in this order, back to back, in the arena too (pooch_finalize)
        ws_wgrad = reinterpret_cast<float *>(base);
        ws_bn = reinterpret_cast<float *>(base + ctx->ws_wgrad_bytes);
        loss_ps = reinterpret_cast<float *>(base + ctx->ws_wgrad_bytes + ctx->ws_bn_bytes);
    }

    float *R(int64_t off) const { return reinterpret_cast<float *>(c->arena + off); }  // resident
    float *D(int64_t off) const
    {
        if (off == OFF_INPUT) return R(c->off_input);
        if (off < 0) return nullptr;
        return reinterpret_cast<float *>(c->arena + c->resident_bytes + off);
    }
    const ParamInfo &P(int node, int which) const { return c->params[c->G.nodes[node].param[which]]; }

    hipError_t forward(int i, int64_t out, int64_t in0, int64_t in1, bool refwd)
    {
        const Graph &G = c->G;
        const Node &nd = G.nodes[i];
        hipStream_t s = c->st[S_COMPUTE];
        switch (nd.op) {
        case OP_CONV:
            return pk::conv_fwd(D(in0), R(P(i, 0).off_val), D(out), conv_geom(G, i, c->in_cdev), s,
                                (!refwd && c->stats_to[i] >= 0) ? ws_bn : nullptr, ws_wgrad);
        case OP_BN: case OP_BNRELU: {
            const int64_t M = nd.numel() / nd.C;
            const bool relu = nd.op == OP_BNRELU;
            // every forward execution moves the running averages; a re-forward uses the saved statistics and does not
            const pk::BnRun run{R(c->off_rmean[i]), R(c->off_rvar[i]), c->bn_decay};
            if (G.apply_into[i] >= 0) {   // applied inside the add + ReLU that consumes it: statistics only
                if (refwd) return hipSuccess;   // nothing to recompute: the statistics are saved, there is no output
                if (c->stats_from[i] >= 0)
                    return pk::bn_stats_from_tiles(ws_bn, c->stats_tiles[i][0], c->stats_tiles[i][1], M, (int)nd.C,
                                                   nd.eps, R(c->off_mean[i]), R(c->off_istd[i]), run, s);
                return pk::bn_stats(D(in0), R(c->off_mean[i]), R(c->off_istd[i]), ws_bn, M, (int)nd.C, nd.eps, run, s);
            }
            if (refwd)
                return pk::bn_apply(D(in0), R(P(i, 0).off_val), R(P(i, 1).off_val), R(c->off_mean[i]), R(c->off_istd[i]),
                                    D(out), M, (int)nd.C, relu, s);
            if (c->stats_from[i] >= 0)   // the convolution that has just run left the statistics per row tile
                return pk::bn_fwd_from_tiles(D(in0), R(P(i, 0).off_val), R(P(i, 1).off_val), D(out), R(c->off_mean[i]),
                                             R(c->off_istd[i]), ws_bn, c->stats_tiles[i][0], c->stats_tiles[i][1], M,
                                             (int)nd.C, nd.eps, relu, run, s);
            return pk::bn_fwd(D(in0), R(P(i, 0).off_val), R(P(i, 1).off_val), D(out), R(c->off_mean[i]), R(c->off_istd[i]),
                              ws_bn, M, (int)nd.C, nd.eps, relu, run, s);
        }
        case OP_RELU: {
            const hipError_t e = pk::relu_fwd(D(in0), D(out), nd.numel(), s);
            return e != hipSuccess ? e : keep_mask(i, out, refwd);
        }
        case OP_ADD: return pk::add_fwd(D(in0), D(in1), D(out), nd.numel(), s);
        case OP_ADDRELU: {
            // inputs whose normalisation is applied here: in0 / in1 then is that layer's input
            const bool ap0 = G.apply_into[nd.in[0]] == i, ap1 = G.apply_into[nd.in[1]] == i;
            hipError_t e;
            if (ap0 || ap1) {
                const int b = nd.in[ap0 ? 0 : 1], b2 = nd.in[1];
                const bool both = ap0 && ap1;
                e = pk::bn_add_relu_fwd(D(ap0 ? in0 : in1), D(ap0 ? in1 : in0), R(P(b, 0).off_val), R(P(b, 1).off_val),
                                        R(c->off_mean[b]), R(c->off_istd[b]), both ? R(P(b2, 0).off_val) : nullptr,
                                        both ? R(P(b2, 1).off_val) : nullptr, both ? R(c->off_mean[b2]) : nullptr,
                                        both ? R(c->off_istd[b2]) : nullptr, D(out), nd.numel() / nd.C, (int)nd.C, s);
            } else {
                e = pk::add_relu_fwd(D(in0), D(in1), D(out), nd.numel(), s);
            }
            return e != hipSuccess ? e : keep_mask(i, out, refwd);
        }
        case OP_MAXPOOL: return pk::maxpool_fwd(D(in0), D(out), pool_geom(G, i), s);
        case OP_GAVGPOOL: {
            const Node &x = G.nodes[nd.in[0]];
            return pk::gavgpool_fwd(D(in0), D(out), (int)x.N, x.sp[0] * x.sp[1] * x.sp[2], (int)x.C, s);
        }
        case OP_FC: {
            hipError_t e = pk::conv_fwd(D(in0), R(P(i, 0).off_val), D(out), conv_geom(G, i, c->in_cdev), s, nullptr, ws_wgrad);
            if (e != hipSuccess) return e;
            return pk::bias_add(D(out), R(P(i, 1).off_val), (int)nd.N, (int)nd.C, s);
        }
        case OP_LOSS: {
            const Node &z = G.nodes[nd.in[0]];
            return pk::softmax_ce_fwd(D(in0), reinterpret_cast<const int32_t *>(c->arena + c->off_labels), loss_ps,
                                      R(c->off_loss), (int)z.N, (int)z.C, s);
        }
        default: return hipErrorInvalidValue;
        }
    }

    // a ReLU that keeps one bit per element for its backward packs them from the output it has just written; a re-forward
    // (the output regenerated as another layer's input) finds the same bits in place already
    hipError_t keep_mask(int i, int64_t out, bool refwd)
    {
        if (c->off_mask[i] < 0 || refwd) return hipSuccess;
        return pk::relu_mask_pack(D(out), reinterpret_cast<uint32_t *>(c->arena + c->off_mask[i]), c->G.nodes[i].numel(), c->st[S_COMPUTE]);
    }

    // one gradient output of an element-wise "pass dy on" (residual add)
    hipError_t pass_on(int64_t dy, int64_t off, int mode, int64_t n)
    {
        hipStream_t s = c->st[S_COMPUTE];
        if (mode == M_WRITE) return pk::copy(D(off), D(dy), n, s);
        if (mode == M_ACC) return pk::accumulate(D(off), D(dy), n, s);
        return hipSuccess;  // none / transferred: the buffer itself changes owner
    }

    hipError_t backward(int i, const int64_t *a)
    {
        const Graph &G = c->G;
        const Node &nd = G.nodes[i];
        hipStream_t s = c->st[S_COMPUTE];
        const int64_t dy = a[0], need = a[1], o0 = a[2], o1 = a[4];
        const int m0 = (int)a[3], m1 = (int)a[5];
        switch (nd.op) {
        case OP_CONV: case OP_FC: {
            const pk::ConvGeom g = conv_geom(G, i, c->in_cdev);
            hipError_t e = pk::conv_wgrad(D(dy), D(need), R(P(i, 0).off_grad), ws_wgrad, g, s);
            if (e != hipSuccess) return e;
            if (nd.op == OP_FC) {
                e = pk::bias_grad(D(dy), R(P(i, 1).off_grad), (int)nd.N, (int)nd.C, s);
                if (e != hipSuccess) return e;
            }
            if (mid) {
                e = hipEventRecord(mid, s);
                if (e != hipSuccess) return e;
            }
            if (m0 == M_NONE) return hipSuccess;
            return pk::conv_dgrad(D(dy), R(P(i, 0).off_val_t), D(o0), g, m0 == M_ACC, s, ws_wgrad);
        }
        case OP_BN: case OP_BNRELU: {
            const int64_t M = nd.numel() / nd.C;
            // no gradient wanted for the input (the network input): dy may be another tensor's gradient too, leave it alone
            float *dx = m0 == M_NONE ? nullptr : D(o0);
            return pk::bn_bwd(D(need), D(dy), R(P(i, 0).off_val), R(P(i, 1).off_val), R(c->off_mean[i]), R(c->off_istd[i]), dx,
                              R(P(i, 0).off_grad), R(P(i, 1).off_grad), ws_bn, M, (int)nd.C, m0 == M_ACC,
                              nd.op == OP_BNRELU, s);
        }
        case OP_ADDRELU: {
            // the masked gradient overwrites dy (one input may take that buffer over); the first
            // input that wants its own copy gets it in the same pass, a second one in a pass of its own
            const int64_t offs[2] = {o0, o1};
            const int modes[2] = {m0, m1};
            int first = -1;
            for (int j = 0; j < 2; ++j)
                if (first < 0 && (modes[j] == M_WRITE || modes[j] == M_ACC)) first = j;
            float *o1 = first < 0 ? nullptr : D(offs[first]);
            const int mode1 = first < 0 ? 0 : (modes[first] == M_WRITE ? 1 : 2);
            hipError_t e = c->off_mask[i] >= 0
                               ? pk::add_relu_bwd_mask(reinterpret_cast<const uint32_t *>(c->arena + c->off_mask[i]), D(dy), o1, mode1, nd.numel(), s)
                               : pk::add_relu_bwd(D(need), D(dy), o1, mode1, nd.numel(), s);
            if (e != hipSuccess) return e;
            for (int j = first + 1; first >= 0 && j < 2; ++j)
                if (modes[j] == M_WRITE || modes[j] == M_ACC) {
                    e = pass_on(dy, offs[j], modes[j], nd.numel());
                    if (e != hipSuccess) return e;
                }
            return hipSuccess;
        }
        case OP_RELU:
            if (m0 == M_NONE) return hipSuccess;
            if (c->off_mask[i] >= 0)
                return pk::relu_bwd_mask(reinterpret_cast<const uint32_t *>(c->arena + c->off_mask[i]), D(dy), D(o0), nd.numel(), m0 == M_ACC, s);
            return pk::relu_bwd(D(need), D(dy), D(o0), nd.numel(), m0 == M_ACC, s);
        case OP_ADD: {
            hipError_t e = pass_on(dy, o0, m0, nd.numel());
            if (e != hipSuccess) return e;
            return pass_on(dy, o1, m1, nd.numel());
        }
        case OP_MAXPOOL:
            if (m0 == M_NONE) return hipSuccess;
            return pk::maxpool_bwd(D(need), D(dy), D(o0), pool_geom(G, i), m0 == M_ACC, s);
        case OP_GAVGPOOL: {
            if (m0 == M_NONE) return hipSuccess;
            const Node &x = G.nodes[nd.in[0]];
            return pk::gavgpool_bwd(D(dy), D(o0), (int)x.N, x.sp[0] * x.sp[1] * x.sp[2], (int)x.C, m0 == M_ACC, s);
        }
        case OP_LOSS: {
            if (m0 == M_NONE) return hipSuccess;
            const Node &z = G.nodes[nd.in[0]];
            return pk::softmax_ce_bwd(D(need), reinterpret_cast<const int32_t *>(c->arena + c->off_labels), D(o0), (int)z.N,
                                      (int)z.C, m0 == M_ACC, s);
        }
        default: return hipErrorInvalidValue;
        }
    }
};

pooch_status ensure_events(pooch_ctx *c, std::vector<hipEvent_t> &pool, size_t n, unsigned flags)
{
    while (pool.size() < n) {
        hipEvent_t e;
        HIPCHK(hipEventCreateWithFlags(&e, flags));
        pool.push_back(e);
    }
    return POOCH_OK;
}

pooch_status copy_out_capture(pooch_ctx *c, int i, const float *dev)
{
    const Node &nd = c->G.nodes[i];
    const int64_t n = nd.numel();
    c->host_tmp.resize((size_t)n);
    HIPCHK(hipStreamSynchronize(c->st[S_COMPUTE]));
    HIPCHK(hipMemcpy(c->host_tmp.data(), dev, (size_t)n * 4, hipMemcpyDeviceToHost));
    act_from_device_layout(c->host_tmp.data(), nd.N, nd.C, nd.sp[0] * nd.sp[1] * nd.sp[2], c->capture[i]);
    return POOCH_OK;
}

// Enqueues a command list.  tm != nullptr: every forward / re-forward / backward / copy command
// is bracketed by timing events on its own stream; profile_refwd additionally runs (and
// times) each layer's re-forward variant right after its forward, on the same buffers.
// A command that follows another on its stream with no wait in between starts at that one's stop
// event instead of recording one of its own (an event between every two kernels cost 2.3 ms per
// step on ResNet-50, 10 % of the step at batch 64; half of them are left).
// Returns at the first failure with whatever was enqueued before it still in flight: run_schedule() cleans up.
pooch_status enqueue_schedule(pooch_ctx *c, const Schedule &S, Timing *tm, bool profile_refwd, bool static_scratch)
{
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (!c->has_batch) return fail(c, POOCH_E_STATE, "no batch: call pooch_set_batch first");
    for (char ok : c->param_set)
        if (!ok) return fail(c, POOCH_E_STATE, "a parameter was never set: call pooch_set_param for every parameter first");
    const size_t swap_bytes = (size_t)S.swap_bytes;
    if (swap_bytes > 0 && (!c->pinned || swap_bytes > c->pinned_bytes)) return fail(c, POOCH_E_BUDGET, "pinned buffer too small");
    pooch_status ps = POOCH_OK;
    if (static_scratch) {   // this path creates nothing: the events were made when the plan was installed
        if (c->sync_events.size() < (size_t)S.n_events) return fail(c, POOCH_E_STATE, "the plan's events do not exist");
    } else {
        ps = ensure_events(c, c->sync_events, (size_t)S.n_events, hipEventDisableTiming);
        if (ps != POOCH_OK) return ps;
    }
    const int64_t cap = (int64_t)c->arena_bytes - c->resident_bytes;
    size_t n_te = 0;
    if (tm) {
        const size_t nc = S.cmds.size();
        tm->start.assign(nc, -1); tm->stop.assign(nc, -1); tm->rstart.assign(nc, -1); tm->rstop.assign(nc, -1);
        tm->mid.assign(nc, -1);
        tm->own_start.assign(nc, 0);
        int last[3] = {-1, -1, -1};     // per stream: the stop event of its latest command, -1 once the stream may have stalled since
        for (size_t k = 0; k < nc; ++k) {
            const Cmd &cm = S.cmds[k];
            const int kind = cm.kind;
            if (kind == K_WAIT) last[cm.id] = -1;
            if (kind == K_REC || kind == K_WAIT) continue;
            const int st = kind <= K_BWD ? S_COMPUTE : (kind == K_OUT ? S_D2H : S_H2D);
            if (last[st] >= 0) {
                tm->start[k] = last[st];
            } else {
                tm->start[k] = (int)n_te++;
                tm->own_start[k] = 1;
            }
            const Op op = kind <= K_BWD ? c->G.nodes[cm.id].op : OP_INPUT;
            if (kind == K_BWD && (op == OP_CONV || op == OP_FC)) tm->mid[k] = (int)n_te++;
            tm->stop[k] = (int)n_te++;
            last[st] = tm->stop[k];
            if (profile_refwd && kind == K_FWD && op != OP_LOSS) {
                tm->rstart[k] = tm->stop[k];
                tm->rstop[k] = (int)n_te++;
                last[st] = tm->rstop[k];
            }
            if (kind == K_FWD && c->capture[cm.id] && op != OP_LOSS) last[st] = -1;   // a blocking copy follows
        }
        ps = ensure_events(c, c->timing_events, n_te, hipEventDefault);
        if (ps != POOCH_OK) return ps;
    }
    Exec X(c, S, static_scratch);
    const Graph &G = c->G;
    auto in_arena = [&](int64_t off, int64_t bytes) { return off == OFF_INPUT || off == OFF_NONE || (off >= 0 && off % ALIGN == 0 && off + bytes <= cap); };
    for (size_t k = 0; k < S.cmds.size(); ++k) {
        const Cmd &cm = S.cmds[k];
        const int stream = cm.kind <= K_BWD ? S_COMPUTE : (cm.kind == K_OUT ? S_D2H : (cm.kind == K_IN ? S_H2D : cm.id));
        if ((int64_t)k == c->fail_at) {
            c->fail_at = -1;
            return fail(c, POOCH_E_HIP, "injected failure at command " + std::to_string(k) + " (pooch_inject_failure)");
        }
        if (tm && tm->own_start[k]) HIPCHK(hipEventRecord(c->timing_events[tm->start[k]], c->st[stream]));
        switch (cm.kind) {
        case K_FWD: case K_REFWD: {
            const int i = cm.id;
            if (!in_arena(cm.a[0], G.bytes[i])) return fail(c, POOCH_E_INVALID, "command outside the arena");
            {
                const hipError_t fe = X.forward(i, cm.a[0], cm.a[1], cm.a[2], cm.kind == K_REFWD);
                if (fe != hipSuccess)
                    return fail(c, POOCH_E_HIP, std::string(cm.kind == K_REFWD ? "re-forward" : "forward") + " of node " + std::to_string(i) +
                                                    " (command " + std::to_string(k) + ", offsets " + std::to_string(cm.a[0]) + " " + std::to_string(cm.a[1]) + " " +
                                                    std::to_string(cm.a[2]) + "): " + hipGetErrorString(fe));
            }
            if (tm && tm->start[k] >= 0) HIPCHK(hipEventRecord(c->timing_events[tm->stop[k]], c->st[stream]));
            if (tm && tm->rstart[k] >= 0) {
                HIPCHK(X.forward(i, cm.a[0], cm.a[1], cm.a[2], true));
                HIPCHK(hipEventRecord(c->timing_events[tm->rstop[k]], c->st[stream]));
            }
            if (cm.kind == K_FWD && c->capture[i] && G.nodes[i].op != OP_LOSS) {
                ps = copy_out_capture(c, i, X.D(cm.a[0]));
                if (ps != POOCH_OK) return ps;
            }
            break;
        }
        case K_BWD: {
            const int i = cm.id;
            for (int j = 0; j < 2; ++j)
                if (cm.a[3 + 2 * j] != M_NONE && !in_arena(cm.a[2 + 2 * j], G.gbytes[G.nodes[i].in[j]]))
                    return fail(c, POOCH_E_INVALID, "command outside the arena");
            X.mid = (tm && tm->mid[k] >= 0) ? c->timing_events[tm->mid[k]] : nullptr;
            {
                const hipError_t be = X.backward(i, cm.a);
                X.mid = nullptr;
                if (be != hipSuccess)
                    return fail(c, POOCH_E_HIP, "backward of node " + std::to_string(i) + " (command " + std::to_string(k) + "): " + hipGetErrorString(be));
            }
            if (tm && tm->start[k] >= 0) HIPCHK(hipEventRecord(c->timing_events[tm->stop[k]], c->st[stream]));
            break;
        }
        case K_OUT: {
            const int64_t bytes = G.nodes[cm.id].numel() * 4;
            if (!in_arena(cm.a[0], bytes) || (size_t)(cm.a[1] + bytes) > c->pinned_bytes) return fail(c, POOCH_E_INVALID, "swap-out outside its buffers");
            HIPCHK(hipMemcpyAsync(c->pinned + cm.a[1], X.D(cm.a[0]), (size_t)bytes, hipMemcpyDeviceToHost, c->st[S_D2H]));
            if (tm) HIPCHK(hipEventRecord(c->timing_events[tm->stop[k]], c->st[stream]));
            break;
        }
        case K_IN: {
            const int64_t bytes = G.nodes[cm.id].numel() * 4;
            if (!in_arena(cm.a[0], bytes) || (size_t)(cm.a[1] + bytes) > c->pinned_bytes) return fail(c, POOCH_E_INVALID, "swap-in outside its buffers");
            HIPCHK(hipMemcpyAsync(X.D(cm.a[0]), c->pinned + cm.a[1], (size_t)bytes, hipMemcpyHostToDevice, c->st[S_H2D]));
            if (tm) HIPCHK(hipEventRecord(c->timing_events[tm->stop[k]], c->st[stream]));
            break;
        }
        case K_REC: HIPCHK(hipEventRecord(c->sync_events[cm.a[0]], c->st[cm.id])); break;
        case K_WAIT: HIPCHK(hipStreamWaitEvent(c->st[cm.id], c->sync_events[cm.a[0]], 0)); break;
        default: return fail(c, POOCH_E_INVALID, "unknown command");
        }
    }
    return POOCH_OK;
}

// Replays a command list and waits for it.  A failure part-way (a HIP call that returns an error, a command that
// does not fit its buffers) leaves commands of the first part queued on up to three streams: they are waited for
// before the error is reported, so that nothing of the failed step is still running when the caller acts on it,
// and the gradients are marked absent (pooch_get_grad / pooch_sgd_update refuse until a step has completed).
// What a later step needs is untouched by a partial one -- parameters, the batch and the plan are only read, and a
// step writes every range of the dynamic region before it reads it -- so the same context can simply step again;
// BN running averages of the layers that did run have moved.
pooch_status run_schedule(pooch_ctx *c, const Schedule &S, Timing *tm, bool profile_refwd, float *loss_out,
                          bool static_scratch = false)
{
    c->has_grads = false;
    pooch_status ps = enqueue_schedule(c, S, tm, profile_refwd, static_scratch);
    hipError_t first = hipSuccess;
    for (int s = 0; s < 3; ++s) {
        const hipError_t e = hipStreamSynchronize(c->st[s]);
        if (first == hipSuccess) first = e;
    }
    if (ps != POOCH_OK) return ps;   // the message of the failure itself stays
    if (first != hipSuccess) return fail(c, POOCH_E_HIP, std::string("hipStreamSynchronize: ") + hipGetErrorString(first));
    if (loss_out) HIPCHK(hipMemcpy(loss_out, c->arena + c->off_loss, 4, hipMemcpyDeviceToHost));
    c->has_grads = true;
    return POOCH_OK;
}

pooch_status elapsed(pooch_ctx *c, int a, int b, double &ms)
{
    float f = 0.f;
    HIPCHK(hipEventElapsedTime(&f, c->timing_events[a], c->timing_events[b]));
    ms = (double)f;
    return POOCH_OK;
}

double median(std::vector<double> &v)
{
    if (v.empty()) return 0.0;
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n % 2 ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
}

int32_t add_node(pooch_ctx *c, const Node &nd)
{
    c->G.nodes.push_back(nd);
    return (int32_t)c->G.nodes.size() - 1;
}

bool valid_tensor(const pooch_ctx *c, int32_t x)
{
    return x >= 0 && x < (int32_t)c->G.nodes.size() && c->G.nodes[x].op != OP_LOSS;
}

#define GRAPH_OPEN(c)                                                           \
    do {                                                                        \
        if (!(c)) return POOCH_E_INVALID;                                       \
        if ((c)->finalized) return fail((c), POOCH_E_STATE, "graph is frozen"); \
    } while (0)

bool window_out(const Node &x, int nspatial, const int *k, const int *stride, const int *pad, Node &nd)
{
    if (nspatial != x.nsp || (nspatial != 2 && nspatial != 3)) return false;
    nd.nsp = nspatial;
    nd.N = x.N;
    for (int d = 0; d < 3; ++d) { nd.k[d] = 1; nd.st[d] = 1; nd.pd[d] = 0; nd.sp[d] = 1; }
    const int o = 3 - nspatial;
    for (int d = 0; d < nspatial; ++d) {
        if (k[d] <= 0 || stride[d] <= 0 || pad[d] < 0) return false;
        nd.k[o + d] = k[d]; nd.st[o + d] = stride[d]; nd.pd[o + d] = pad[d];
        const int64_t in = x.sp[o + d];
        if (in + 2 * pad[d] < k[d]) return false;
        nd.sp[o + d] = (in + 2 * pad[d] - k[d]) / stride[d] + 1;
    }
    return true;
}

pooch_status install(pooch_ctx *c, const std::vector<uint8_t> &cls, bool ahead, double predicted)
{
    Schedule S;
    std::string why;
    const int64_t cap = (int64_t)c->arena_bytes - c->resident_bytes;
    const int64_t pinned_cap = c->arena ? (int64_t)c->pinned_bytes : -1;
    if (!build_schedule(c->G, cls, cap, ahead, pinned_cap, S, &why)) return fail(c, POOCH_E_BUDGET, why);
    if (c->arena) {   // the plan's events exist from here on: a step creates none
        const pooch_status ps = ensure_events(c, c->sync_events, (size_t)S.n_events, hipEventDisableTiming);
        if (ps != POOCH_OK) return ps;
    }
    c->sched = std::move(S);
    c->cls = cls;
    c->ahead = ahead;
    c->has_plan = true;
    c->predicted_ms = predicted;
    return POOCH_OK;
}

Profile zero_profile(const Graph &G)
{
    Profile P;
    P.t_fwd.assign(G.n(), 0.0); P.t_bwd.assign(G.n(), 0.0); P.t_refwd.assign(G.n(), 0.0);
    P.t_out.assign(G.fmaps.size(), 0.0); P.t_in.assign(G.fmaps.size(), 0.0);
    P.valid = true;
    return P;
}

bool valid_classes(const pooch_ctx *c, const uint8_t *cls)
{
    for (size_t k = 0; k < c->G.fmaps.size(); ++k)
        if (cls[k] > CLS_RECOMPUTE) return false;
    return true;
}

}  // namespace

extern "C" {

pooch_status pooch_create(void *arena, size_t arena_bytes, void *pinned_host, size_t pinned_bytes, void *stream_compute,
                          void *stream_d2h, void *stream_h2d, pooch_ctx **out)
{
    if (!out) return POOCH_E_INVALID;
    *out = nullptr;
    if (arena && ((uintptr_t)arena % ALIGN != 0)) return POOCH_E_INVALID;
    if (!pinned_host && pinned_bytes != 0) return POOCH_E_INVALID;
    pooch_ctx *c = new (std::nothrow) pooch_ctx();
    if (!c) return POOCH_E_INVALID;
    c->arena = static_cast<char *>(arena);
    // whole 256-byte units only: ranges carved from the top of the dynamic region start at (capacity - size), which
    // has to be as aligned as every other offset (a budget of an odd number of bytes gave a convolution an odd address)
    c->arena_bytes = arena_bytes / ALIGN * ALIGN;
    c->pinned = static_cast<char *>(pinned_host);
    c->pinned_bytes = pinned_bytes;
    c->st[0] = static_cast<hipStream_t>(stream_compute);
    c->st[1] = static_cast<hipStream_t>(stream_d2h);
    c->st[2] = static_cast<hipStream_t>(stream_h2d);
    if (arena) {
        // the GPU that holds the arena also holds a copy of the static scratch array: its address there, looked up once
        // per device (pooch_step_static_scratch); a failure is reported by that entry point, not here
        hipPointerAttribute_t attr;
        void *ptr = nullptr;
        if (hipPointerGetAttributes(&attr, arena) == hipSuccess && static_scratch_for(attr.device, &ptr) == hipSuccess)
            c->static_scratch = static_cast<char *>(ptr);
        else
            (void)hipGetLastError();
    }
    *out = c;
    return POOCH_OK;
}

void pooch_destroy(pooch_ctx *c)
{
    if (!c) return;
    for (hipEvent_t e : c->sync_events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->timing_events) (void)hipEventDestroy(e);
    delete c;
}

const char *pooch_last_error(pooch_ctx *c) { return c ? c->err.c_str() : "null context"; }

int32_t pooch_input(pooch_ctx *c, const int64_t *dims, int ndim)
{
    GRAPH_OPEN(c);
    if (!dims || (ndim != 4 && ndim != 5) || !c->G.nodes.empty()) return fail(c, POOCH_E_INVALID, "input: bad dims or not the first node");
    Node nd;
    nd.op = OP_INPUT;
    nd.nsp = ndim - 2;
    nd.N = dims[0];
    nd.C = dims[1];
    for (int d = 0; d < nd.nsp; ++d) nd.sp[3 - nd.nsp + d] = dims[2 + d];
    if (nd.N <= 0 || nd.C <= 0 || nd.sp[0] <= 0 || nd.sp[1] <= 0 || nd.sp[2] <= 0) return fail(c, POOCH_E_INVALID, "input: non-positive size");
    return add_node(c, nd);
}

int32_t pooch_conv(pooch_ctx *c, int32_t x, int cout, const int *k, const int *stride, const int *pad, int nspatial)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, x) || cout <= 0 || !k || !stride || !pad) return fail(c, POOCH_E_INVALID, "conv: bad argument");
    Node nd;
    nd.op = OP_CONV;
    if (!window_out(c->G.nodes[x], nspatial, k, stride, pad, nd)) return fail(c, POOCH_E_INVALID, "conv: bad geometry");
    nd.C = cout;
    nd.in[0] = x;
    nd.nin = 1;
    return add_node(c, nd);
}

int32_t pooch_bn(pooch_ctx *c, int32_t x, float eps)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, x) || !(eps >= 0.f)) return fail(c, POOCH_E_INVALID, "bn: bad argument");
    Node nd = c->G.nodes[x];
    nd.op = OP_BN;
    nd.in[0] = x; nd.in[1] = -1;
    nd.nin = 1;
    nd.eps = eps;
    nd.param[0] = nd.param[1] = -1;
    return add_node(c, nd);
}

int32_t pooch_relu(pooch_ctx *c, int32_t x)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, x)) return fail(c, POOCH_E_INVALID, "relu: bad argument");
    Node nd = c->G.nodes[x];
    nd.op = OP_RELU;
    nd.in[0] = x; nd.in[1] = -1;
    nd.nin = 1;
    nd.param[0] = nd.param[1] = -1;
    return add_node(c, nd);
}

int32_t pooch_add(pooch_ctx *c, int32_t a, int32_t b)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, a) || !valid_tensor(c, b)) return fail(c, POOCH_E_INVALID, "add: bad argument");
    if (a == b) return fail(c, POOCH_E_INVALID, "add: the two inputs must be different tensors");
    const Node &A = c->G.nodes[a], &B = c->G.nodes[b];
    if (A.N != B.N || A.C != B.C || A.sp[0] != B.sp[0] || A.sp[1] != B.sp[1] || A.sp[2] != B.sp[2] || A.nsp != B.nsp)
        return fail(c, POOCH_E_INVALID, "add: shapes differ");
    Node nd = A;
    nd.op = OP_ADD;
    nd.in[0] = a; nd.in[1] = b;
    nd.nin = 2;
    nd.param[0] = nd.param[1] = -1;
    return add_node(c, nd);
}

int32_t pooch_maxpool(pooch_ctx *c, int32_t x, const int *k, const int *stride, const int *pad, int nspatial)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, x) || !k || !stride || !pad) return fail(c, POOCH_E_INVALID, "maxpool: bad argument");
    Node nd;
    nd.op = OP_MAXPOOL;
    if (!window_out(c->G.nodes[x], nspatial, k, stride, pad, nd)) return fail(c, POOCH_E_INVALID, "maxpool: bad geometry");
    for (int d = 0; d < nspatial; ++d)
        if (pad[d] >= k[d]) return fail(c, POOCH_E_INVALID, "maxpool: padding must be smaller than the window");
    nd.C = c->G.nodes[x].C;
    nd.in[0] = x;
    nd.nin = 1;
    return add_node(c, nd);
}

int32_t pooch_gavgpool(pooch_ctx *c, int32_t x)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, x)) return fail(c, POOCH_E_INVALID, "gavgpool: bad argument");
    Node nd;
    nd.op = OP_GAVGPOOL;
    nd.nsp = c->G.nodes[x].nsp;
    nd.N = c->G.nodes[x].N;
    nd.C = c->G.nodes[x].C;
    nd.in[0] = x;
    nd.nin = 1;
    return add_node(c, nd);
}

int32_t pooch_fc(pooch_ctx *c, int32_t x, int nout)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, x) || nout <= 0) return fail(c, POOCH_E_INVALID, "fc: bad argument");
    Node nd;
    nd.op = OP_FC;
    nd.nsp = c->G.nodes[x].nsp;
    nd.N = c->G.nodes[x].N;
    nd.C = nout;
    nd.in[0] = x;
    nd.nin = 1;
    return add_node(c, nd);
}

int32_t pooch_softmax_ce(pooch_ctx *c, int32_t logits)
{
    GRAPH_OPEN(c);
    if (!valid_tensor(c, logits)) return fail(c, POOCH_E_INVALID, "softmax_ce: bad argument");
    const Node &z = c->G.nodes[logits];
    if (z.sp[0] * z.sp[1] * z.sp[2] != 1) return fail(c, POOCH_E_INVALID, "softmax_ce: logits must be N x classes");
    Node nd;
    nd.op = OP_LOSS;
    nd.N = 1; nd.C = 1;
    nd.in[0] = logits;
    nd.nin = 1;
    return add_node(c, nd);
}

pooch_status pooch_set_fusion(pooch_ctx *c, int enable)
{
    GRAPH_OPEN(c);
    c->G.fuse = enable != 0;
    return POOCH_OK;
}

pooch_status pooch_set_relu_masks(pooch_ctx *c, int enable)
{
    GRAPH_OPEN(c);
    c->G.masks = enable != 0;
    return POOCH_OK;
}

int32_t pooch_node_keeps_mask(pooch_ctx *c, int32_t id)
{
    if (!c || !c->finalized) return POOCH_E_STATE;
    if (id < 0 || id >= c->G.n()) return POOCH_E_INVALID;
    return c->G.mask_only[id] ? 1 : 0;
}

int32_t pooch_node_fused(pooch_ctx *c, int32_t id)
{
    if (!c || !c->finalized) return POOCH_E_STATE;
    if (id < 0 || id >= c->G.n()) return POOCH_E_INVALID;
    return c->G.fused_into[id] >= 0 ? c->G.fused_into[id] : c->G.apply_into[id];
}

int32_t pooch_bn_stats_source(pooch_ctx *c, int32_t id)
{
    if (!c || !c->finalized) return POOCH_E_STATE;
    if (id < 0 || id >= c->G.n()) return POOCH_E_INVALID;
    return c->stats_from[id];
}

pooch_status pooch_finalize(pooch_ctx *c)
{
    GRAPH_OPEN(c);
    Graph &G = c->G;
    const std::string bad = G.analyze();
    if (!bad.empty()) return fail(c, POOCH_E_INVALID, bad);
    const int n = G.n();
    int64_t off = 0;
    auto take = [&](int64_t bytes) { const int64_t o = off; off += round_up(bytes); return o; };
    c->in_cdev = (int)G.nodes[0].C;
    if (G.nodes[0].C < 4) {   // one to three input channels: stored with zero channels up to four (16-byte taps)
        bool only_convs = true;
        for (int u : G.consumers[0]) only_convs = only_convs && G.nodes[u].op == OP_CONV;
        if (only_convs) c->in_cdev = 4;
    }
    c->off_input = take(G.nodes[0].numel() / G.nodes[0].C * c->in_cdev * 4);
    c->off_labels = take(G.nodes[0].N * 4);
    c->off_mean.assign(n, -1);
    c->off_istd.assign(n, -1);
    c->off_rmean.assign(n, -1);
    c->off_rvar.assign(n, -1);
    c->off_mask.assign(n, -1);
    c->params.clear();
    size_t ws_wgrad = 0, ws_bn = 0;
    for (int i = 0; i < n; ++i) {
        Node &nd = G.nodes[i];
        if (G.mask_only[i]) c->off_mask[i] = take((int64_t)pk::relu_mask_bytes(nd.numel()));
        if (nd.op == OP_CONV || nd.op == OP_FC) {
            const pk::ConvGeom g = conv_geom(G, i, c->in_cdev);
            // the conv kernels index rows and reduction lengths with 32 bits
            const int64_t lim = ((int64_t)1 << 31) - 4096;
            if (g.rows_in() >= lim || g.rows_out() >= lim || g.taps() * std::max(g.C, g.K) >= lim)
                return fail(c, POOCH_E_INVALID, "conv/fc: tensor too large for the kernels' 32-bit row index");
            const int64_t dev_numel = (int64_t)g.K * g.C * g.taps();
            const int64_t numel = (int64_t)g.K * G.nodes[nd.in[0]].C * g.taps();
            ParamInfo p{i, 0, numel, dev_numel, take(dev_numel * 4), take(dev_numel * 4), take(dev_numel * 4)};
            nd.param[0] = (int)c->params.size();
            c->params.push_back(p);
            // one workspace serves the filter gradient's split-K partials and the split reductions of small forward /
            // data-gradient GEMMs: the launches that use it are serialised on the compute stream
            ws_wgrad = std::max({ws_wgrad, pk::conv_wgrad_workspace(g), pk::conv_fwd_workspace(g), pk::conv_dgrad_workspace(g)});
            if (nd.op == OP_FC) {
                ParamInfo b{i, 1, nd.C, nd.C, take(nd.C * 4), -1, take(nd.C * 4)};
                nd.param[1] = (int)c->params.size();
                c->params.push_back(b);
            }
        } else if (nd.op == OP_BN || (nd.op == OP_DEAD && G.nodes[G.fused_into[i]].op == OP_BNRELU)) {
            for (int w = 0; w < 2; ++w) {
                ParamInfo p{i, w, nd.C, nd.C, take(nd.C * 4), -1, take(nd.C * 4)};
                nd.param[w] = (int)c->params.size();
                c->params.push_back(p);
            }
            c->off_mean[i] = take(nd.C * 4);
            c->off_istd[i] = take(nd.C * 4);
            c->off_rmean[i] = take(nd.C * 4);
            c->off_rvar[i] = take(nd.C * 4);
            ws_bn = std::max(ws_bn, pk::bn_workspace_floats(nd.numel() / nd.C, (int)nd.C) * 4);
        } else if (nd.op == OP_LOSS) {
            c->nclasses = (int)G.nodes[nd.in[0]].C;
        }
    }
    for (int i = 0; i < n; ++i) {
        const int j = G.fused_into[i];
        if (j >= 0 && G.nodes[j].op == OP_BNRELU) {
            G.nodes[j].param[0] = G.nodes[i].param[0];
            G.nodes[j].param[1] = G.nodes[i].param[1];
            c->off_mean[j] = c->off_mean[i];
            c->off_istd[j] = c->off_istd[i];
            c->off_rmean[j] = c->off_rmean[i];
            c->off_rvar[j] = c->off_rvar[i];
        }
    }
    // convolutions followed directly by their batch normalisation hand it the statistics
    c->stats_to.assign(n, -1);
    c->stats_from.assign(n, -1);
    c->stats_tiles.assign(n, std::array<int, 2>{0, 0});
    if (getenv("POOCH_NO_CONV_STATS") == nullptr) {
        const float *aligned = reinterpret_cast<const float *>((uintptr_t)ALIGN);   // every tensor is ALIGN-byte aligned
        for (int i = 0; i < n; ++i) {
            if (G.nodes[i].op != OP_CONV) continue;
            int j = i + 1;
            while (j < n && G.nodes[j].op == OP_DEAD) ++j;
            if (j >= n || (G.nodes[j].op != OP_BN && G.nodes[j].op != OP_BNRELU) || G.nodes[j].in[0] != i) continue;
            int tiles_m = 0, rows = 0;
            if (!pk::conv_fwd_bn_tiles(aligned, aligned, conv_geom(G, i, c->in_cdev), &tiles_m, &rows)) continue;
            c->stats_to[i] = j;
            c->stats_from[j] = i;
            c->stats_tiles[j] = {tiles_m, rows};
            ws_bn = std::max(ws_bn, pk::bn_tiles_workspace_floats(tiles_m, (int)G.nodes[i].C) * 4);
        }
    }
    // the kernels' scratch: three ranges back to back (Exec relies on the order)
    c->ws_wgrad_bytes = round_up((int64_t)ws_wgrad);
    c->ws_bn_bytes = round_up((int64_t)ws_bn);
    c->loss_ps_bytes = round_up(G.nodes[0].N * 4);
    c->off_ws_wgrad = take(c->ws_wgrad_bytes);
    c->off_ws_bn = take(c->ws_bn_bytes);
    c->off_loss_ps = take(c->loss_ps_bytes);
    c->off_loss = take(4);
    c->resident_bytes = off;
    if ((size_t)off > c->arena_bytes) return fail(c, POOCH_E_BUDGET, "the resident region alone exceeds the arena");
    c->capture.assign(n, nullptr);
    if (c->arena) {   // running averages start at mean 0, variance 1
        for (int i = 0; i < n; ++i) {
            if (c->off_rmean[i] < 0 || G.nodes[i].op == OP_DEAD) continue;
            const std::vector<float> zero((size_t)G.nodes[i].C, 0.f), one((size_t)G.nodes[i].C, 1.f);
            HIPCHK(hipMemcpy(c->arena + c->off_rmean[i], zero.data(), zero.size() * 4, hipMemcpyHostToDevice));
            HIPCHK(hipMemcpy(c->arena + c->off_rvar[i], one.data(), one.size() * 4, hipMemcpyHostToDevice));
        }
    }
    c->param_set.assign(c->params.size(), 0);
    c->finalized = true;
    return POOCH_OK;
}

#define NEED_FINAL(c)                                                                     \
    do {                                                                                  \
        if (!(c)) return POOCH_E_INVALID;                                                 \
        if (!(c)->finalized) return fail((c), POOCH_E_STATE, "graph is not finalized");  \
    } while (0)

int32_t pooch_num_params(pooch_ctx *c)
{
    NEED_FINAL(c);
    return (int32_t)c->params.size();
}

pooch_status pooch_param_info(pooch_ctx *c, int32_t i, int64_t *numel, int32_t *node)
{
    NEED_FINAL(c);
    if (i < 0 || i >= (int32_t)c->params.size()) return fail(c, POOCH_E_INVALID, "parameter index out of range");
    if (numel) *numel = c->params[i].numel;
    if (node) *node = c->params[i].node;
    return POOCH_OK;
}

pooch_status pooch_set_param(pooch_ctx *c, int32_t i, const float *host)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (i < 0 || i >= (int32_t)c->params.size() || !host) return fail(c, POOCH_E_INVALID, "set_param: bad argument");
    const ParamInfo &p = c->params[i];
    if (p.off_val_t < 0) {
        HIPCHK(hipMemcpy(c->arena + p.off_val, host, (size_t)p.numel * 4, hipMemcpyHostToDevice));
        c->param_set[i] = 1;
        return POOCH_OK;
    }
    const pk::ConvGeom g = conv_geom(c->G, p.node, c->in_cdev);
    std::vector<float> krc((size_t)p.dev_numel, 0.f), crk((size_t)p.dev_numel, 0.f);
    const int64_t Clog = p.numel / ((int64_t)g.K * g.taps());
    filter_to_device_layouts(host, g.K, Clog, g.C, g.taps(), krc.data(), crk.data());
    HIPCHK(hipMemcpy(c->arena + p.off_val, krc.data(), (size_t)p.dev_numel * 4, hipMemcpyHostToDevice));
    HIPCHK(hipMemcpy(c->arena + p.off_val_t, crk.data(), (size_t)p.dev_numel * 4, hipMemcpyHostToDevice));
    c->param_set[i] = 1;
    return POOCH_OK;
}

pooch_status pooch_get_grad(pooch_ctx *c, int32_t i, float *host)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (i < 0 || i >= (int32_t)c->params.size() || !host) return fail(c, POOCH_E_INVALID, "get_grad: bad argument");
    if (!c->has_grads) return fail(c, POOCH_E_STATE, "get_grad: no step has run");
    const ParamInfo &p = c->params[i];
    if (p.off_val_t < 0) {
        HIPCHK(hipMemcpy(host, c->arena + p.off_grad, (size_t)p.numel * 4, hipMemcpyDeviceToHost));
        return POOCH_OK;
    }
    const pk::ConvGeom g = conv_geom(c->G, p.node, c->in_cdev);
    std::vector<float> krc((size_t)p.dev_numel);
    HIPCHK(hipMemcpy(krc.data(), c->arena + p.off_grad, (size_t)p.dev_numel * 4, hipMemcpyDeviceToHost));
    filter_from_device_layout(krc.data(), g.K, p.numel / ((int64_t)g.K * g.taps()), g.C, g.taps(), host);
    return POOCH_OK;
}

pooch_status pooch_set_batch(pooch_ctx *c, const float *x_host, const int32_t *labels_host)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (!x_host || !labels_host) return fail(c, POOCH_E_INVALID, "set_batch: null pointer");
    const Node &in = c->G.nodes[0];
    for (int64_t n = 0; n < in.N; ++n)
        if (labels_host[n] < 0 || labels_host[n] >= c->nclasses) return fail(c, POOCH_E_INVALID, "set_batch: label out of range");
    std::vector<float> tmp((size_t)(in.numel() / in.C * c->in_cdev), 0.f);
    act_to_device_layout(x_host, in.N, in.C, c->in_cdev, in.sp[0] * in.sp[1] * in.sp[2], tmp.data());
    HIPCHK(hipMemcpy(c->arena + c->off_input, tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(hipMemcpy(c->arena + c->off_labels, labels_host, (size_t)in.N * 4, hipMemcpyHostToDevice));
    c->has_batch = true;
    return POOCH_OK;
}

pooch_status pooch_capture_tensor(pooch_ctx *c, int32_t id, float *host)
{
    NEED_FINAL(c);
    if (id <= 0 || id >= c->G.n() || c->G.nodes[id].op == OP_LOSS) return fail(c, POOCH_E_INVALID, "capture: not a layer output");
    if (c->G.nodes[id].op == OP_DEAD || c->G.apply_into[id] >= 0)
        return fail(c, POOCH_E_STATE, "capture: this layer is fused into its consumer, its output is never materialised");
    c->capture[id] = host;
    return POOCH_OK;
}

pooch_status pooch_inject_failure(pooch_ctx *c, int64_t command_index)
{
    if (!c) return POOCH_E_INVALID;
    c->fail_at = command_index < 0 ? -1 : command_index;
    return POOCH_OK;
}

pooch_status pooch_get_bn_stats(pooch_ctx *c, int32_t node, float *mean, float *istd)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (node < 0 || node >= c->G.n() || c->off_mean[node] < 0) return fail(c, POOCH_E_INVALID, "not a bn node");
    const size_t bytes = (size_t)c->G.nodes[node].C * 4;
    if (mean) HIPCHK(hipMemcpy(mean, c->arena + c->off_mean[node], bytes, hipMemcpyDeviceToHost));
    if (istd) HIPCHK(hipMemcpy(istd, c->arena + c->off_istd[node], bytes, hipMemcpyDeviceToHost));
    return POOCH_OK;
}

pooch_status pooch_get_bn_running(pooch_ctx *c, int32_t node, float *mean, float *var)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (node < 0 || node >= c->G.n() || c->off_rmean[node] < 0) return fail(c, POOCH_E_INVALID, "not a bn node");
    const size_t bytes = (size_t)c->G.nodes[node].C * 4;
    if (mean) HIPCHK(hipMemcpy(mean, c->arena + c->off_rmean[node], bytes, hipMemcpyDeviceToHost));
    if (var) HIPCHK(hipMemcpy(var, c->arena + c->off_rvar[node], bytes, hipMemcpyDeviceToHost));
    return POOCH_OK;
}

pooch_status pooch_set_bn_running(pooch_ctx *c, int32_t node, const float *mean, const float *var)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (node < 0 || node >= c->G.n() || c->off_rmean[node] < 0) return fail(c, POOCH_E_INVALID, "not a bn node");
    const size_t bytes = (size_t)c->G.nodes[node].C * 4;
    if (mean) HIPCHK(hipMemcpy(c->arena + c->off_rmean[node], mean, bytes, hipMemcpyHostToDevice));
    if (var) HIPCHK(hipMemcpy(c->arena + c->off_rvar[node], var, bytes, hipMemcpyHostToDevice));
    return POOCH_OK;
}

pooch_status pooch_set_bn_decay(pooch_ctx *c, float decay)
{
    if (!c) return POOCH_E_INVALID;
    if (!(decay >= 0.f && decay <= 1.f)) return fail(c, POOCH_E_INVALID, "bn decay must lie in [0, 1]");
    c->bn_decay = decay;
    return POOCH_OK;
}

int32_t pooch_num_nodes(pooch_ctx *c)
{
    if (!c) return POOCH_E_INVALID;
    return (int32_t)c->G.nodes.size();
}

int32_t pooch_num_fmaps(pooch_ctx *c)
{
    NEED_FINAL(c);
    return (int32_t)c->G.fmaps.size();
}

pooch_status pooch_fmap_info(pooch_ctx *c, int32_t i, size_t *bytes, int32_t *producer)
{
    NEED_FINAL(c);
    if (i < 0 || i >= (int32_t)c->G.fmaps.size()) return fail(c, POOCH_E_INVALID, "feature-map index out of range");
    if (bytes) *bytes = (size_t)c->G.bytes[c->G.fmaps[i]];
    if (producer) *producer = c->G.fmaps[i];
    return POOCH_OK;
}

size_t pooch_resident_bytes(pooch_ctx *c) { return (c && c->finalized) ? (size_t)c->resident_bytes : 0; }

}  // extern "C" (reopened below)

namespace {

pooch_status profile_begin(pooch_ctx *c)
{
    const Graph &G = c->G;
    const std::vector<uint8_t> allswap(G.fmaps.size(), CLS_SWAP);
    std::string why;
    c->prof_sched = Schedule();
    if (!build_schedule(G, allswap, (int64_t)c->arena_bytes - c->resident_bytes, true, (int64_t)c->pinned_bytes, c->prof_sched, &why))
        return fail(c, POOCH_E_BUDGET, "profiling runs every map as swap and that does not fit: " + why);
    c->prof_sched_ok = true;
    c->smp_f.assign(G.n(), {}); c->smp_b.assign(G.n(), {}); c->smp_r.assign(G.n(), {});
    c->smp_o.assign(G.fmaps.size(), {}); c->smp_i.assign(G.fmaps.size(), {});
    return POOCH_OK;
}

// one all-swap step; timed: every command's duration is added to the samples
pooch_status profile_one(pooch_ctx *c, bool timed, float *loss_out)
{
    const Graph &G = c->G;
    const Schedule &S = c->prof_sched;
    Timing tm;
    pooch_status ps = run_schedule(c, S, timed ? &tm : nullptr, timed, loss_out);
    if (ps != POOCH_OK || !timed) return ps;
    for (size_t k = 0; k < S.cmds.size(); ++k) {
        if (tm.start[k] < 0) continue;
        const Cmd &cm = S.cmds[k];
        double ms;
        ps = elapsed(c, tm.start[k], tm.stop[k], ms);
        if (ps != POOCH_OK) return ps;
        switch (cm.kind) {
        case K_FWD: c->smp_f[cm.id].push_back(ms); break;
        case K_REFWD: c->smp_r[cm.id].push_back(ms); break;
        case K_BWD: c->smp_b[cm.id].push_back(ms); break;
        case K_OUT: c->smp_o[G.fidx[cm.id]].push_back(ms); break;
        case K_IN: c->smp_i[G.fidx[cm.id]].push_back(ms); break;
        default: break;
        }
        if (tm.rstart[k] >= 0) {
            ps = elapsed(c, tm.rstart[k], tm.rstop[k], ms);
            if (ps != POOCH_OK) return ps;
            c->smp_r[cm.id].push_back(ms);
        }
    }
    return POOCH_OK;
}

// a profiling iteration failed: no half-gathered samples and no profiling schedule are left behind (the profile
// measured or injected earlier, if any, stays valid)
void profile_abort(pooch_ctx *c)
{
    c->prof_sched_ok = false;
    c->prof_sched = Schedule();
    c->smp_f.clear(); c->smp_b.clear(); c->smp_r.clear(); c->smp_o.clear(); c->smp_i.clear();
}

pooch_status profile_end(pooch_ctx *c)
{
    const int n = c->G.n();
    const size_t nf = c->G.fmaps.size();
    bool any = false;
    for (int i = 1; i < n; ++i) any = any || !c->smp_f[i].empty();
    if (!any) return fail(c, POOCH_E_NOPROFILE, "no timed profiling step was run");
    Profile P;
    P.t_fwd.resize(n); P.t_bwd.resize(n); P.t_refwd.resize(n); P.t_out.resize(nf); P.t_in.resize(nf);
    for (int i = 0; i < n; ++i) { P.t_fwd[i] = median(c->smp_f[i]); P.t_bwd[i] = median(c->smp_b[i]); P.t_refwd[i] = median(c->smp_r[i]); }
    for (size_t k = 0; k < nf; ++k) { P.t_out[k] = median(c->smp_o[k]); P.t_in[k] = median(c->smp_i[k]); }
    P.valid = true;
    c->prof = P;
    c->profile_newer_than_plan = c->has_plan;
    c->prof_sched_ok = false;
    return POOCH_OK;
}

}  // namespace

extern "C" {

pooch_status pooch_profile(pooch_ctx *c, int warmup, int iters)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (warmup < 0 || iters <= 0) return fail(c, POOCH_E_INVALID, "profile: bad iteration counts");
    pooch_status ps = profile_begin(c);
    if (ps != POOCH_OK) return ps;
    for (int it = 0; it < warmup + iters; ++it) {
        ps = profile_one(c, it >= warmup, nullptr);
        if (ps != POOCH_OK) {
            profile_abort(c);
            return ps;
        }
    }
    return profile_end(c);
}

pooch_status pooch_profile_step(pooch_ctx *c, int timed, float *loss_out)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (!c->prof_sched_ok) {
        const pooch_status ps = profile_begin(c);
        if (ps != POOCH_OK) return ps;
    }
    const pooch_status ps = profile_one(c, timed != 0, loss_out);
    if (ps != POOCH_OK) profile_abort(c);   // the samples gathered so far are dropped with the failed iteration
    return ps;
}

pooch_status pooch_finish_profile(pooch_ctx *c)
{
    NEED_FINAL(c);
    if (!c->prof_sched_ok) return fail(c, POOCH_E_STATE, "finish_profile: no profiling step was run");
    return profile_end(c);
}

pooch_status pooch_sgd_update(pooch_ctx *c, float lr)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (!(lr == lr)) return fail(c, POOCH_E_INVALID, "sgd_update: learning rate is NaN");
    if (!c->has_grads) return fail(c, POOCH_E_STATE, "sgd_update: no step has run");
    hipStream_t s = c->st[S_COMPUTE];
    for (const ParamInfo &p : c->params) {
        float *val = reinterpret_cast<float *>(c->arena + p.off_val);
        HIPCHK(pk::sgd_update(val, reinterpret_cast<const float *>(c->arena + p.off_grad), lr, p.dev_numel, s));
        if (p.off_val_t >= 0) {
            const pk::ConvGeom g = conv_geom(c->G, p.node, c->in_cdev);
            HIPCHK(pk::filter_transpose(val, reinterpret_cast<float *>(c->arena + p.off_val_t), g.K, g.taps(), g.C, s));
        }
    }
    HIPCHK(hipStreamSynchronize(s));
    return POOCH_OK;
}

pooch_status pooch_get_param(pooch_ctx *c, int32_t i, float *host)
{
    NEED_FINAL(c);
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (i < 0 || i >= (int32_t)c->params.size() || !host) return fail(c, POOCH_E_INVALID, "get_param: bad argument");
    const ParamInfo &p = c->params[i];
    if (p.off_val_t < 0) {
        HIPCHK(hipMemcpy(host, c->arena + p.off_val, (size_t)p.numel * 4, hipMemcpyDeviceToHost));
        return POOCH_OK;
    }
    const pk::ConvGeom g = conv_geom(c->G, p.node, c->in_cdev);
    std::vector<float> krc((size_t)p.dev_numel);
    HIPCHK(hipMemcpy(krc.data(), c->arena + p.off_val, (size_t)p.dev_numel * 4, hipMemcpyDeviceToHost));
    filter_from_device_layout(krc.data(), g.K, p.numel / ((int64_t)g.K * g.taps()), g.C, g.taps(), host);
    return POOCH_OK;
}

pooch_status pooch_get_profile(pooch_ctx *c, double *t_fwd, double *t_bwd, double *t_refwd, double *t_out, double *t_in)
{
    NEED_FINAL(c);
    if (!c->prof.valid) return fail(c, POOCH_E_NOPROFILE, "no profile");
    const Profile &P = c->prof;
    if (t_fwd) std::copy(P.t_fwd.begin(), P.t_fwd.end(), t_fwd);
    if (t_bwd) std::copy(P.t_bwd.begin(), P.t_bwd.end(), t_bwd);
    if (t_refwd) std::copy(P.t_refwd.begin(), P.t_refwd.end(), t_refwd);
    if (t_out) std::copy(P.t_out.begin(), P.t_out.end(), t_out);
    if (t_in) std::copy(P.t_in.begin(), P.t_in.end(), t_in);
    return POOCH_OK;
}

pooch_status pooch_set_profile(pooch_ctx *c, const double *t_fwd, const double *t_bwd, const double *t_refwd, const double *t_out,
                               const double *t_in)
{
    NEED_FINAL(c);
    if (!t_fwd || !t_bwd || !t_refwd || !t_out || !t_in) return fail(c, POOCH_E_INVALID, "set_profile: null pointer");
    const int n = c->G.n();
    const size_t nf = c->G.fmaps.size();
    for (int i = 0; i < n; ++i)
        if (!(t_fwd[i] >= 0.0) || !(t_bwd[i] >= 0.0) || !(t_refwd[i] >= 0.0)) return fail(c, POOCH_E_INVALID, "set_profile: negative or NaN duration");
    for (size_t k = 0; k < nf; ++k)
        if (!(t_out[k] >= 0.0) || !(t_in[k] >= 0.0)) return fail(c, POOCH_E_INVALID, "set_profile: negative or NaN duration");
    Profile P;
    P.t_fwd.assign(t_fwd, t_fwd + n); P.t_bwd.assign(t_bwd, t_bwd + n); P.t_refwd.assign(t_refwd, t_refwd + n);
    P.t_out.assign(t_out, t_out + nf); P.t_in.assign(t_in, t_in + nf);
    P.valid = true;
    c->prof = P;
    c->profile_newer_than_plan = c->has_plan;
    return POOCH_OK;
}

pooch_status pooch_plan(pooch_ctx *c, int mode, int max_bruteforce_bits, double *predicted_ms)
{
    NEED_FINAL(c);
    if (mode < POOCH_MODE_INCORE || mode > POOCH_MODE_SUPERNEURONS) return fail(c, POOCH_E_INVALID, "plan: unknown mode");
    if (!c->prof.valid && mode >= POOCH_MODE_SWAPOPT && mode != POOCH_MODE_SUPERNEURONS) return fail(c, POOCH_E_NOPROFILE, "plan: the search needs a profile");
    const Profile zero = c->prof.valid ? Profile() : zero_profile(c->G);
    const Profile &P = c->prof.valid ? c->prof : zero;
    int bits = max_bruteforce_bits <= 0 ? 10 : max_bruteforce_bits;
    if (bits > 20) bits = 20;
    const int64_t cap = (int64_t)c->arena_bytes - c->resident_bytes;
    Planner pl(c->G, P, cap, c->arena ? (int64_t)c->pinned_bytes : -1, bits);
    pl.restarts = c->restarts;
    // a plan made from an earlier state of the profile competes as the refine search's starting point
    const std::vector<uint8_t> seed = c->cls;
    if (mode == POOCH_MODE_REFINE && c->has_plan && c->ahead && c->profile_newer_than_plan) pl.seed = &seed;
    std::vector<uint8_t> cls;
    double T = 0.0;
    bool ahead = true;
    const bool ok = pl.plan(mode, cls, T, ahead);
    c->evals = pl.evals;
    if (!ok) return fail(c, POOCH_E_BUDGET, "plan: not even the safest plan of this mode fits the budget");
    const pooch_status ps = install(c, cls, ahead, T);
    if (ps != POOCH_OK) return ps;
    c->profile_newer_than_plan = false;
    if (predicted_ms) *predicted_ms = T;
    return POOCH_OK;
}

pooch_status pooch_set_search_effort(pooch_ctx *c, int restarts)
{
    if (!c) return POOCH_E_INVALID;
    if (restarts < 0 || restarts > 100000) return fail(c, POOCH_E_INVALID, "search effort out of range");
    c->restarts = restarts;
    return POOCH_OK;
}

pooch_status pooch_get_plan(pooch_ctx *c, uint8_t *cls)
{
    NEED_FINAL(c);
    if (!c->has_plan) return fail(c, POOCH_E_STATE, "no plan installed");
    if (!cls) return fail(c, POOCH_E_INVALID, "get_plan: null pointer");
    std::copy(c->cls.begin(), c->cls.end(), cls);
    return POOCH_OK;
}

pooch_status pooch_set_plan(pooch_ctx *c, const uint8_t *cls, int sched)
{
    NEED_FINAL(c);
    if (!cls || !valid_classes(c, cls)) return fail(c, POOCH_E_INVALID, "set_plan: bad classification");
    const std::vector<uint8_t> v(cls, cls + c->G.fmaps.size());
    double T = 0.0;
    if (c->prof.valid) {
        Schedule S;
        if (build_schedule(c->G, v, (int64_t)c->arena_bytes - c->resident_bytes, sched != 0,
                           c->arena ? (int64_t)c->pinned_bytes : -1, S))
            T = simulate(c->G, S, c->prof).T;
    }
    return install(c, v, sched != 0, T);
}

pooch_status pooch_simulate(pooch_ctx *c, const uint8_t *cls, int sched, double *step_ms, size_t *peak_bytes)
{
    NEED_FINAL(c);
    if (!cls || !valid_classes(c, cls)) return fail(c, POOCH_E_INVALID, "simulate: bad classification");
    const std::vector<uint8_t> v(cls, cls + c->G.fmaps.size());
    Schedule S;
    std::string why;
    if (!build_schedule(c->G, v, (int64_t)c->arena_bytes - c->resident_bytes, sched != 0, c->arena ? (int64_t)c->pinned_bytes : -1, S, &why))
        return fail(c, POOCH_E_BUDGET, why);
    if (peak_bytes) *peak_bytes = (size_t)S.peak;
    if (step_ms) {
        if (!c->prof.valid) return fail(c, POOCH_E_NOPROFILE, "simulate: no profile");
        *step_ms = simulate(c->G, S, c->prof).T;
    }
    return POOCH_OK;
}

int64_t pooch_plan_evaluations(pooch_ctx *c) { return c ? c->evals : 0; }

pooch_status pooch_get_overhead_sets(pooch_ctx *c, uint8_t *in_LO, uint8_t *in_LI)
{
    NEED_FINAL(c);
    if (!c->prof.valid) return fail(c, POOCH_E_NOPROFILE, "overhead sets: no profile");
    const std::vector<uint8_t> allswap(c->G.fmaps.size(), CLS_SWAP);
    Schedule S;
    std::string why;
    if (!build_schedule(c->G, allswap, (int64_t)c->arena_bytes - c->resident_bytes, true, c->arena ? (int64_t)c->pinned_bytes : -1, S, &why))
        return fail(c, POOCH_E_BUDGET, why);
    const SimResult sr = simulate(c->G, S, c->prof);
    const size_t nf = c->G.fmaps.size();
    if (in_LO) { std::fill(in_LO, in_LO + nf, 0); for (int t : sr.LO) in_LO[c->G.fidx[t]] = 1; }
    if (in_LI) { std::fill(in_LI, in_LI + nf, 0); for (int t : sr.LI) in_LI[c->G.fidx[t]] = 1; }
    return POOCH_OK;
}

pooch_status pooch_get_commands(pooch_ctx *c, int64_t *rows, int64_t max_rows, int64_t *nrows)
{
    NEED_FINAL(c);
    if (!c->has_plan) return fail(c, POOCH_E_STATE, "no plan installed");
    const int64_t n = (int64_t)c->sched.cmds.size();
    if (nrows) *nrows = n;
    if (!rows) return POOCH_OK;
    if (max_rows < n) return fail(c, POOCH_E_INVALID, "get_commands: buffer too small");
    for (int64_t k = 0; k < n; ++k) {
        const Cmd &cm = c->sched.cmds[k];
        int64_t *r = rows + 8 * k;
        r[0] = cm.kind; r[1] = cm.id;
        for (int j = 0; j < 6; ++j) r[2 + j] = cm.a[j];
    }
    return POOCH_OK;
}

pooch_status pooch_step(pooch_ctx *c, float *loss_out)
{
    NEED_FINAL(c);
    if (!c->has_plan) return fail(c, POOCH_E_STATE, "step: no plan installed");
    const auto t0 = std::chrono::steady_clock::now();
    const pooch_status ps = run_schedule(c, c->sched, nullptr, false, loss_out);
    c->last_step_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return ps;
}

pooch_status pooch_step_static_scratch(pooch_ctx *c, float *loss_out)
{
    NEED_FINAL(c);
    const int64_t need = c->ws_wgrad_bytes + c->ws_bn_bytes + c->loss_ps_bytes;
    if ((size_t)need > STATIC_SCRATCH_BYTES)
        return fail(c, POOCH_E_BUDGET, "step_static_scratch: this network's kernels need " + std::to_string(need) +
                                           " bytes of scratch, the static buffer holds " + std::to_string(STATIC_SCRATCH_BYTES));
    if (!c->arena) return fail(c, POOCH_E_STATE, "planning-only context (no arena)");
    if (!c->has_plan) return fail(c, POOCH_E_STATE, "step: no plan installed");
    if (!c->static_scratch) return fail(c, POOCH_E_HIP, "step_static_scratch: the static scratch array's device address is not available");
    const auto t0 = std::chrono::steady_clock::now();
    const pooch_status ps = run_schedule(c, c->sched, nullptr, false, loss_out, true);
    c->last_step_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return ps;
}

pooch_status pooch_get_stats(pooch_ctx *c, pooch_stats *st)
{
    NEED_FINAL(c);
    if (!st) return fail(c, POOCH_E_INVALID, "get_stats: null pointer");
    std::memset(st, 0, sizeof(*st));
    st->resident_bytes = (uint64_t)c->resident_bytes;
    st->arena_bytes = (uint64_t)c->arena_bytes;
    st->scratch_bytes = (uint64_t)(c->ws_wgrad_bytes + c->ws_bn_bytes + c->loss_ps_bytes);
    if (!c->has_plan) return POOCH_OK;
    st->step_ms = c->last_step_ms;
    st->predicted_ms = c->predicted_ms;
    uint64_t out_b = 0, in_b = 0;
    for (const Cmd &cm : c->sched.cmds) {
        if (cm.kind == K_OUT) out_b += (uint64_t)c->G.nodes[cm.id].numel() * 4;
        if (cm.kind == K_IN) in_b += (uint64_t)c->G.nodes[cm.id].numel() * 4;
    }
    st->swap_out_bytes = out_b;
    st->swap_in_bytes = in_b;
    st->peak_bytes = (uint64_t)c->sched.peak;
    st->extent_bytes = (uint64_t)c->sched.extent;
    for (uint8_t k : c->cls) {
        if (k == CLS_KEEP) st->n_keep++;
        else if (k == CLS_SWAP) st->n_swap++;
        else st->n_recompute++;
    }
    st->n_commands = (int32_t)c->sched.cmds.size();
    st->n_refwd = c->sched.n_refwd;
    return POOCH_OK;
}

pooch_status pooch_step_timed(pooch_ctx *c, float *loss_out, double *ms_fwd, double *ms_bwd, double *ms_refwd, double *ms_bwd_filter)
{
    NEED_FINAL(c);
    if (!c->has_plan) return fail(c, POOCH_E_STATE, "step: no plan installed");
    Timing tm;
    pooch_status ps = run_schedule(c, c->sched, &tm, false, loss_out);
    if (ps != POOCH_OK) return ps;
    const int n = c->G.n();
    if (ms_fwd) std::fill(ms_fwd, ms_fwd + n, 0.0);
    if (ms_bwd) std::fill(ms_bwd, ms_bwd + n, 0.0);
    if (ms_refwd) std::fill(ms_refwd, ms_refwd + n, 0.0);
    if (ms_bwd_filter) std::fill(ms_bwd_filter, ms_bwd_filter + n, 0.0);
    for (size_t k = 0; k < c->sched.cmds.size(); ++k) {
        const Cmd &cm = c->sched.cmds[k];
        if (cm.kind > K_BWD) continue;
        double ms;
        ps = elapsed(c, tm.start[k], tm.stop[k], ms);
        if (ps != POOCH_OK) return ps;
        double *dst = cm.kind == K_FWD ? ms_fwd : (cm.kind == K_BWD ? ms_bwd : ms_refwd);
        if (dst) dst[cm.id] += ms;
        if (ms_bwd_filter && tm.mid[k] >= 0) {
            ps = elapsed(c, tm.start[k], tm.mid[k], ms);
            if (ps != POOCH_OK) return ps;
            ms_bwd_filter[cm.id] += ms;
        }
    }
    return POOCH_OK;
}

pooch_status pooch_refine_profile(pooch_ctx *c, int iters, float *loss_out)
{
    NEED_FINAL(c);
    if (!c->has_plan) return fail(c, POOCH_E_STATE, "refine_profile: no plan installed");
    if (!c->prof.valid) return fail(c, POOCH_E_NOPROFILE, "refine_profile: no profile to refine");
    if (iters < 1) return fail(c, POOCH_E_INVALID, "refine_profile: iters must be positive");
    const int n = c->G.n();
    std::vector<std::vector<double>> f(n), b(n), r(n);
    for (int it = 0; it < iters; ++it) {
        Timing tm;
        pooch_status ps = run_schedule(c, c->sched, &tm, false, loss_out);
        if (ps != POOCH_OK) return ps;
        for (size_t k = 0; k < c->sched.cmds.size(); ++k) {
            const Cmd &cm = c->sched.cmds[k];
            if (cm.kind > K_BWD) continue;
            double ms;
            ps = elapsed(c, tm.start[k], tm.stop[k], ms);
            if (ps != POOCH_OK) return ps;
            (cm.kind == K_FWD ? f : (cm.kind == K_BWD ? b : r))[cm.id].push_back(ms);
        }
    }
    for (int i = 0; i < n; ++i) {
        if (!f[i].empty()) c->prof.t_fwd[i] = median(f[i]);
        if (!b[i].empty()) c->prof.t_bwd[i] = median(b[i]);
        if (!r[i].empty()) c->prof.t_refwd[i] = median(r[i]);
    }
    c->profile_newer_than_plan = true;
    return POOCH_OK;
}

const char *pooch_node_kernel(pooch_ctx *c, int32_t node, int part)
{
    if (!c || !c->finalized || node < 0 || node >= c->G.n() || part < 0 || part > 3) return "";
    const Op op = c->G.nodes[node].op;
    if (op != OP_CONV && op != OP_FC) return "";
    const pk::ConvGeom g = conv_geom(c->G, node, c->in_cdev);
    if (part == 0) return pk::conv_fwd_kernel(g, c->stats_to[node] >= 0);
    if (part == 3) return pk::conv_fwd_kernel(g, false);
    return part == 1 ? pk::conv_dgrad_kernel(g) : pk::conv_wgrad_kernel(g);
}

pooch_status pooch_measure_link(pooch_ctx *c, size_t bytes, int iters, double *d2h_gbs, double *h2d_gbs)
{
    NEED_FINAL(c);
    if (!c->arena || !c->pinned) return fail(c, POOCH_E_STATE, "measure_link needs an arena and a pinned buffer");
    const size_t dyn = c->arena_bytes - (size_t)c->resident_bytes;
    if (bytes == 0 || iters <= 0 || bytes > c->pinned_bytes || bytes > dyn) return fail(c, POOCH_E_INVALID, "measure_link: bad size");
    pooch_status ps = ensure_events(c, c->timing_events, 2, hipEventDefault);
    if (ps != POOCH_OK) return ps;
    char *dev = c->arena + c->resident_bytes;
    for (int dir = 0; dir < 2; ++dir) {
        hipStream_t s = c->st[dir == 0 ? S_D2H : S_H2D];
        // one untimed copy first
        if (dir == 0) HIPCHK(hipMemcpyAsync(c->pinned, dev, bytes, hipMemcpyDeviceToHost, s));
        else HIPCHK(hipMemcpyAsync(dev, c->pinned, bytes, hipMemcpyHostToDevice, s));
        HIPCHK(hipEventRecord(c->timing_events[0], s));
        for (int it = 0; it < iters; ++it) {
            if (dir == 0) HIPCHK(hipMemcpyAsync(c->pinned, dev, bytes, hipMemcpyDeviceToHost, s));
            else HIPCHK(hipMemcpyAsync(dev, c->pinned, bytes, hipMemcpyHostToDevice, s));
        }
        HIPCHK(hipEventRecord(c->timing_events[1], s));
        HIPCHK(hipStreamSynchronize(s));
        double ms;
        ps = elapsed(c, 0, 1, ms);
        if (ps != POOCH_OK) return ps;
        const double gbs = (double)bytes * iters / (ms * 1e-3) / 1e9;
        if (dir == 0 && d2h_gbs) *d2h_gbs = gbs;
        if (dir == 1 && h2d_gbs) *h2d_gbs = gbs;
    }
    return POOCH_OK;
}

}  // extern "C"
