// Host-side core of the out-of-core training step: layer graph, feature-map set, static
// schedule inside a fixed arena, timeline simulation and the classification search.
// Pure C++ (no HIP): everything here runs without a GPU.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace pooch {

enum Op : int { OP_INPUT = 0, OP_CONV, OP_BN, OP_RELU, OP_ADD, OP_MAXPOOL, OP_GAVGPOOL, OP_FC, OP_LOSS,
                // produced by fusion: BN / add executed inside the ReLU that is their only consumer; the BN /
                // add node itself becomes OP_DEAD (no output, no commands)
                OP_BNRELU, OP_ADDRELU, OP_DEAD };

enum : int { CLS_KEEP = 0, CLS_SWAP = 1, CLS_RECOMPUTE = 2 };

// command kinds of the replayed list
enum : int { K_FWD = 0, K_REFWD = 1, K_BWD = 2, K_OUT = 3, K_IN = 4, K_REC = 5, K_WAIT = 6 };
enum : int { S_COMPUTE = 0, S_D2H = 1, S_H2D = 2 };
// how a backward command produces the gradient of one of its inputs
enum : int { M_NONE = 0, M_WRITE = 1, M_ACC = 2, M_TRANSFER = 3 };
constexpr int64_t OFF_INPUT = -2;  // the network input sits in the resident region
constexpr int64_t OFF_NONE = -1;
constexpr int64_t ALIGN = 256;

struct Node {
    Op op = OP_INPUT;
    int in[2] = {-1, -1};
    int nin = 0;
    int nsp = 2;                 // spatial rank (2 or 3) of this node's output
    int64_t N = 0, C = 0;        // output batch / channels
    int64_t sp[3] = {1, 1, 1};   // output D,H,W (D = 1 for 2-d; all 1 after gavgpool / fc)
    int k[3] = {1, 1, 1}, st[3] = {1, 1, 1}, pd[3] = {0, 0, 0};
    float eps = 0.f;
    int param[2] = {-1, -1};     // indices into the parameter list
    int64_t numel() const { return N * C * sp[0] * sp[1] * sp[2]; }
};

struct Graph {
    std::vector<Node> nodes;
    bool fuse = true;
    // filled by analyze()
    std::vector<int> fused_into;                // BN / add node -> the ReLU node that executes it, or -1
    std::vector<int64_t> bytes;                 // arena bytes of each node's output (0 for the loss)
    std::vector<int64_t> gbytes;                // ... of its gradient: a full tensor also where the output is never written
    // A BN whose only consumer is the add of an add+ReLU node is applied inside that node's forward
    // kernel (apply_into[bn] = the add+ReLU node; the first such input only).  The BN node stays: its
    // forward is the statistics alone and writes no tensor (zero bytes), its backward is unchanged and
    // still receives the gradient along the edge from the add.  Hence two edge sets: inputs / consumers
    // carry gradients; finputs / fconsumers say what a forward kernel reads (the add+ReLU reads the
    // BN's input in place of the BN's output) and decide how long tensors live (last_consumer).
    std::vector<int> apply_into;
    std::vector<std::vector<int>> inputs;       // as given (may repeat)
    std::vector<std::vector<int>> consumers;    // consumers along the gradient edges, ascending, unique
    std::vector<std::vector<int>> finputs, fconsumers;
    std::vector<int> last_consumer;
    std::vector<std::vector<int>> needs;        // tensors the backward of a node reads
    // masks: a ReLU (or add + ReLU) whose output no OTHER layer's backward reads keeps one bit per element -- was the
    // output positive -- for its own backward instead of the output (mask_only[node]); the output then is no feature map
    bool masks = false;
    std::vector<char> mask_only;
    std::vector<int> fmaps;                     // tensor id of every feature map, ascending
    std::vector<int> fidx;                      // tensor id -> feature-map index or -1
    int n() const { return (int)nodes.size(); }
    // returns an empty string or a description of what is wrong with the graph
    std::string analyze();
};

struct Cmd {
    int32_t kind;
    int32_t id;      // node (F/R/B), tensor (O/I) or stream (REC/WAIT)
    int64_t a[6];    // F/R: out,in0,in1 | B: dy,need,o0,m0,o1,m1 | O/I: dev_off,pinned_off | REC/WAIT: event
};

struct Schedule {
    std::vector<Cmd> cmds;
    int64_t peak = 0, extent = 0, swap_bytes = 0;
    int n_events = 0, n_refwd = 0;
    std::vector<int> d2h_event;     // completion event of swap-out k
    std::vector<int> d2h_map;       // tensor of swap-out k
    std::vector<int> arrive_event;  // per tensor: event recorded after its swap-in, or -1
};

// false: the classification does not fit (arena or pinned buffer); why receives the reason
bool build_schedule(const Graph &G, const std::vector<uint8_t> &cls, int64_t cap, bool ahead, int64_t pinned_cap,
                    Schedule &out, std::string *why = nullptr);

struct Profile {
    std::vector<double> t_fwd, t_bwd, t_refwd;  // per node, ms
    std::vector<double> t_out, t_in;            // per feature map, ms
    bool valid = false;
};

struct SimResult {
    double T = 0.0;
    std::vector<int> LO, LI;  // tensor ids, ascending
};
SimResult simulate(const Graph &G, const Schedule &S, const Profile &P);

enum : int { MODE_INCORE = 0, MODE_SWAPALL_NOSCHED = 1, MODE_SWAPALL = 2, MODE_SWAPOPT = 3, MODE_POOCH = 4, MODE_REFINE = 5, MODE_SUPERNEURONS = 6 };

struct Planner {
    const Graph &G;
    const Profile &P;
    int64_t cap, pinned_cap;
    int max_bits;
    int restarts = 8;  // perturbed restarts of the local search in refine()
    // refine mode: a classification that competes with the two-step plan as the search's starting point
    const std::vector<uint8_t> *seed = nullptr;
    int64_t evals = 0;
    std::vector<int> LO, LI;
    Planner(const Graph &g, const Profile &p, int64_t cap_, int64_t pinned_cap_, int max_bits_)
        : G(g), P(p), cap(cap_), pinned_cap(pinned_cap_), max_bits(max_bits_) {}
    // simulated step time of a classification, or a negative number if it does not fit
    double evaluate(const std::vector<uint8_t> &cls, bool ahead = true, int64_t cap_override = -1);
    // false: not even the safest plan of this mode fits
    bool plan(int mode, std::vector<uint8_t> &cls, double &T, bool &ahead);
    void step1(const std::vector<uint8_t> &allswap, double T_all, std::vector<uint8_t> &best, double &best_T);
    void step2(std::vector<uint8_t> &cls, double &T0);
    void descend(std::vector<uint8_t> &cls, double &T0);
    void refine(std::vector<uint8_t> &cls, double &T0);
};

}  // namespace pooch
