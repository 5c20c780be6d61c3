// Host side of the packed-training library: the C ABI of include/pack.h, the planner that turns
// K layer lists into a static launch sequence over lists of problems, and weight I/O.
//
// The packed model of the paper (Section 2.2: outputs concatenated; Section 3.4: one shared input;
// Section 3.2: smaller batches are slices of the shared batch) is represented as a plan, not as a
// literal concatenated graph: slot s of the plan holds layer s of every member that has one, and
// each slot is executed by one launch per kernel kind over a list of per-member problems.
// Members therefore never exchange data, which is what makes packing lossless (Section 3.1).
#include "../../include/pack.h"
#include "pack_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <system_error>
#include <thread>
#include <vector>

using namespace packk;

namespace {

thread_local std::string g_err;

pack_status fail(pack_status s, const std::string& msg) {
    g_err = msg;
    return s;
}

#define HIP_TRY(expr, status)                                                             \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess)                                                             \
            return fail(status, std::string(#expr) + ": " + hipGetErrorString(e_));      \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

enum NodeKind { NODE_LINEAR = 0, NODE_CONV = 1, NODE_GAP = 2 };

struct TensorInfo {
    int n = 0, h = 0, w = 0, c = 0;
    bool is_input = false;
    bool f32 = false;        // logits are stored as float whatever the pack dtype
    int act_out = 0;         // ActKind the tensor was produced through: gradients written to it take its derivative
    bool needs_grad = false;
    bool grad_written = false;
    int ld_dz = 0;           // leading dimension of dz when padded (logits), 0 = c
    // planning state: the gradient that reaches this tensor through a residual shortcut and is added
    // by the input-gradient product of the block's first convolution instead of a kernel of its own
    const void* sc_dz = nullptr;
    int sc_h = 0, sc_w = 0, sc_c = 0;
    bool sc_down = false;
    void* act = nullptr;
    void* dz = nullptr;
    size_t elems() const { return (size_t)n * h * w * c; }
};

struct NodeInfo {
    int kind = 0;
    int in_t = -1, out_t = -1;
    int out = 0, stride = 1;
    int act = 0;             // ActKind fused into the layer
    int res_src = -1;        // tensor index of the shortcut source, -1 if none
    bool res_down = false;
    size_t w_off = 0, b_off = 0;   // element offsets into the parameter arena
    size_t w_elems = 0;      // weights in the public blob
    size_t w_arena = 0;      // weights in the arena (rows padded to `kp` for im2col convolutions)
    int kp = 0;              // > 0: first-layer convolution executed over the shared im2col buffer
    int im2col_idx = -1;     // which shared buffer (pack_ctx::im2col)
    int fan_in = 0;
    size_t blob_off = 0;     // float offset of W in the member's public blob
    bool has_wt = false;     // convolution with an input gradient: a transposed copy of W is kept per step
    size_t wt_off = 0;       // element offset of that copy in pack_ctx::wt
};

struct ModelInfo {
    bool vacant = false;             // slot without a member (freed, not yet loaded again)
    std::vector<pack_layer> layers;  // the member as given, kept to plan it again when the pack changes
    std::vector<TensorInfo> tensors;
    std::vector<NodeInfo> nodes;
    int batch = 0, C = 0;
    size_t n_params = 0;             // floats in the public blob
    size_t arena_begin = 0, arena_end = 0;
    int* pred = nullptr;
    float* loss = nullptr;
    bool fused_head = false;         // classifier head (last linear layer, loss, its input gradient) runs in one kernel
    float* head_partial = nullptr;   // per-block loss sums of that kernel
};

enum LaunchKind { L_GEMM, L_REDUCE, L_CE, L_GAP_FWD, L_GAP_BWD, L_SHORTCUT, L_SGD, L_IM2COL, L_WTRANS, L_HEAD };

struct Launch {
    int kind = 0, mode = 0;
    int tile_cfg = 0;       // GEMM launches: index into GEMM_TILE_M / GEMM_TILE_N
    size_t desc_off = 0;    // byte offset of the problem array in the descriptor buffer
    size_t map_off = 0;     // byte offset of the tile / block map
    int n = 0;              // grid size
    double flops = 0.0;     // GEMM launches: 2 * rows * columns * reduction, summed over the launch's problems
    double bytes = 0.0;     // GEMM launches: operands once + results once (+ the fused update's weight traffic)
};

}  // namespace

namespace packk {
std::string conv_dw_halo_walk(bool bf16, bool wide, const GemmProb& p, const TileRef& tr, long long a_bytes, long long b_bytes,
                              bool every_chunk, long long* loads, long long* frag_reads);
std::string conv_rows_halo_walk(bool bf16, bool narrow, bool dx, const GemmProb& p, const TileRef& tr, long long a_bytes,
                                long long* loads, long long* frag_reads);
std::string gemm_fetch_walk(bool bf16, int mode, int bm, int bn, const GemmProb& p, const TileRef& tr, unsigned long long* a_lo,
                            unsigned long long* a_hi, unsigned long long* b_lo, unsigned long long* b_hi, long long* loads);
// for the library's other source files: records the text pack_last_error returns
pack_status set_error(pack_status s, const std::string& msg) { return fail(s, msg); }
}  // namespace packk

struct pack_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    bool bf16 = false;
    int K = 0;
    pack_input_spec in{};
    std::vector<ModelInfo> models;
    float* master = nullptr;     // fp32 parameter arena
    float* grad = nullptr;       // same layout
    void* shadow = nullptr;      // bf16 copy of the arena (bf16 packs)
    size_t arena_elems = 0;
    // optimisers other than SGD (all SGD: none of this is allocated or launched)
    std::vector<pack_opt_spec> opt;      // per member
    std::vector<long long> opt_t;        // steps taken per member
    bool any_opt = false;
    float* opt_m = nullptr;              // arena-shaped: momentum / Adagrad accumulator / Adam first moment
    float* opt_v = nullptr;              // arena-shaped: Adam second moment
    OptStatic* opt_params = nullptr;     // device, [K]
    void* wt = nullptr;          // per-step transposed copies [Cin][9][Cout] of convolution weights (operand type)
    long long* seg_end = nullptr;
    char* slab = nullptr;        // activations, gradients wrt activations, loss, predictions
    size_t slab_bytes = 0;
    char* workspace = nullptr;   // partial sums of split reductions
    size_t workspace_bytes = 0;
    char* desc = nullptr;        // problem descriptors and block maps
    size_t desc_bytes = 0;
    int* err_flag = nullptr;
    float* loss_all = nullptr;   // [K]
    void* zeros = nullptr;       // 256 bytes of zeros inside the slab (never written)
    std::vector<Im2colProb> im2col;   // shared-input loaders, one per first-layer stride in use
    bool own_input = false;           // members read their own block of the step's input instead of one shared batch
    bool fused = false;               // all members use plain SGD: the update is applied in the weight-gradient kernels
    bool keep_grads = false;          // fused packs: store the gradients as well (pack_read_grads)
    size_t head_desc_off = 0;         // problem table of the classifier-head launch
    int n_heads = 0;
    std::vector<long long> im2col_xoff;   // byte offset of each loader's source in the step's input
    std::vector<Launch> plan;
    size_t device_bytes = 0;
    // per-launch timing (off unless pack_profile_start was called)
    bool profiling = false;
    int profile_which = -1;
    int profile_every = 1;       // time the chosen launch in every n-th step only
    long long profile_step = 0;  // steps since pack_profile_start
    struct Stamp { int launch; hipEvent_t t0, t1; };
    std::vector<Stamp> stamps;
    // planning without a device (pack_plan_check): allocations hand out made-up addresses, nothing is
    // uploaded, and the problem tables stay on the host
    bool dry = false;
    uintptr_t dry_next = (uintptr_t)1 << 44;
    std::vector<std::pair<uintptr_t, size_t>> dry_regions;
    std::vector<char> desc_host;
};

namespace {

// ---- counter-based initialisation: value = hash(seed, member, tensor, index) -> uniform ---------
inline uint64_t splitmix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
inline float uniform_pm(uint64_t seed, uint64_t member, uint64_t tensor, uint64_t idx, float bound) {
    const uint64_t h = splitmix64(splitmix64(splitmix64(seed ^ (member << 32)) ^ tensor) ^ idx);
    const double u = (double)(h >> 11) * (1.0 / 9007199254740992.0);   // [0,1)
    return (float)((2.0 * u - 1.0) * bound);
}
inline float round_to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    std::memcpy(&f, &u, 4);
    return f;
}

// ---- public blob <-> arena layout ----------------------------------------------------------------
// linear: identical ([out][in]).  conv: blob [Cout][Cin][3][3]  <->  arena [Cout][3][3][Cin].
void blob_to_arena(const ModelInfo& m, const float* blob, std::vector<float>& arena) {
    arena.assign(m.arena_end - m.arena_begin, 0.f);
    for (const NodeInfo& nd : m.nodes) {
        if (nd.kind == NODE_GAP) continue;
        float* W = arena.data() + (nd.w_off - m.arena_begin);
        float* b = arena.data() + (nd.b_off - m.arena_begin);
        const float* src = blob + nd.blob_off;
        if (nd.kind == NODE_LINEAR) {
            std::memcpy(W, src, nd.w_elems * sizeof(float));
        } else {
            const int cin = nd.fan_in / 9;
            const size_t row = nd.kp ? (size_t)nd.kp : (size_t)nd.fan_in;   // padding stays zero
            for (int o = 0; o < nd.out; ++o)
                for (int c = 0; c < cin; ++c)
                    for (int t = 0; t < 9; ++t)
                        W[(size_t)o * row + (size_t)t * cin + c] = src[((size_t)o * cin + c) * 9 + t];
        }
        std::memcpy(b, src + nd.w_elems, (size_t)nd.out * sizeof(float));
    }
}

void arena_to_blob(const ModelInfo& m, const std::vector<float>& arena, float* blob) {
    for (const NodeInfo& nd : m.nodes) {
        if (nd.kind == NODE_GAP) continue;
        const float* W = arena.data() + (nd.w_off - m.arena_begin);
        const float* b = arena.data() + (nd.b_off - m.arena_begin);
        float* dst = blob + nd.blob_off;
        if (nd.kind == NODE_LINEAR) {
            std::memcpy(dst, W, nd.w_elems * sizeof(float));
        } else {
            const int cin = nd.fan_in / 9;
            const size_t row = nd.kp ? (size_t)nd.kp : (size_t)nd.fan_in;
            for (int o = 0; o < nd.out; ++o)
                for (int c = 0; c < cin; ++c)
                    for (int t = 0; t < 9; ++t)
                        dst[((size_t)o * cin + c) * 9 + t] = W[(size_t)o * row + (size_t)t * cin + c];
        }
        std::memcpy(dst + nd.w_elems, b, (size_t)nd.out * sizeof(float));
    }
}

// ---- parse one member's layer list -----------------------------------------------------------------
pack_status parse_model(const pack_input_spec& in, const pack_model_spec& spec, int k, ModelInfo& m) {
    const std::string who = "member " + std::to_string(k) + ": ";
    if (!spec.layers || spec.n_layers < 1) return fail(PACK_EINVAL, who + "empty layer list");
    if (spec.batch < 1 || spec.batch > in.B) return fail(PACK_EINVAL, who + "batch outside [1, B]");
    m.batch = spec.batch;
    m.layers.assign(spec.layers, spec.layers + spec.n_layers);
    TensorInfo t0;
    t0.n = spec.batch; t0.h = in.in_h; t0.w = in.in_w; t0.c = in.in_c; t0.is_input = true;
    m.tensors.push_back(t0);
    int cur = 0;
    std::vector<int> res_stack;
    size_t blob_off = 0;
    for (int i = 0; i < spec.n_layers; ++i) {
        const pack_layer& L = spec.layers[i];
        const int next_op = (i + 1 < spec.n_layers) ? spec.layers[i + 1].op : -1;
        const TensorInfo src = m.tensors[cur];
        switch (L.op) {
            case PACK_LINEAR:
            case PACK_CONV3X3: {
                if (L.out < 1) return fail(PACK_EINVAL, who + "layer width < 1");
                NodeInfo nd;
                TensorInfo o;
                o.n = src.n;
                nd.in_t = cur;
                nd.out = L.out;
                if (L.op == PACK_LINEAR) {
                    nd.kind = NODE_LINEAR;
                    nd.fan_in = src.h * src.w * src.c;
                    o.h = o.w = 1;
                } else {
                    if (L.stride != 1 && L.stride != 2) return fail(PACK_EINVAL, who + "conv stride must be 1 or 2");
                    nd.kind = NODE_CONV;
                    nd.stride = L.stride;
                    nd.fan_in = 9 * src.c;
                    o.h = (src.h - 1) / L.stride + 1;   // = floor((h + 2 - 3) / s) + 1
                    o.w = (src.w - 1) / L.stride + 1;
                }
                o.c = L.out;
                nd.w_elems = (size_t)L.out * nd.fan_in;
                nd.w_arena = nd.w_elems;
                if (L.op == PACK_CONV3X3 && src.is_input && nd.fan_in <= 32) {
                    nd.kp = 32;   // few input channels: run over the shared im2col buffer
                    nd.w_arena = (size_t)L.out * nd.kp;
                }
                nd.blob_off = blob_off;
                blob_off += nd.w_elems + L.out;
                if (next_op == PACK_RELU || next_op == PACK_SIGMOID || next_op == PACK_TANH || next_op == PACK_LEAKY_RELU) {
                    nd.act = next_op == PACK_RELU ? ACT_RELU : next_op == PACK_SIGMOID ? ACT_SIGMOID
                           : next_op == PACK_TANH ? ACT_TANH : ACT_LEAKY;
                    ++i;
                } else if (next_op == PACK_RES_END) {
                    if (L.op != PACK_CONV3X3) return fail(PACK_ESHAPE, who + "RES_END must directly follow a CONV3X3");
                    if (res_stack.empty()) return fail(PACK_ESHAPE, who + "RES_END without RES_BEGIN");
                    nd.res_src = res_stack.back();
                    res_stack.pop_back();
                    const TensorInfo& s = m.tensors[nd.res_src];
                    if (s.h == o.h && s.w == o.w && s.c == o.c) {
                        nd.res_down = false;
                    } else if ((s.h + 1) / 2 == o.h && (s.w + 1) / 2 == o.w && s.c <= o.c) {
                        nd.res_down = true;
                    } else {
                        return fail(PACK_ESHAPE, who + "shortcut shapes neither agree nor halve");
                    }
                    nd.act = ACT_RELU;
                    ++i;
                }
                o.act_out = nd.act;
                m.tensors.push_back(o);
                nd.out_t = (int)m.tensors.size() - 1;
                m.nodes.push_back(nd);
                cur = nd.out_t;
                break;
            }
            case PACK_GAP: {
                if (src.is_input) return fail(PACK_ESHAPE, who + "GAP directly on the input is not supported");
                NodeInfo nd;
                nd.kind = NODE_GAP;
                nd.in_t = cur;
                TensorInfo o;
                o.n = src.n; o.h = o.w = 1; o.c = src.c;
                m.tensors.push_back(o);
                nd.out_t = (int)m.tensors.size() - 1;
                m.nodes.push_back(nd);
                cur = nd.out_t;
                break;
            }
            case PACK_RES_BEGIN:
                res_stack.push_back(cur);
                break;
            case PACK_RELU:
            case PACK_SIGMOID:
            case PACK_TANH:
            case PACK_LEAKY_RELU:
                return fail(PACK_ESHAPE, who + "an activation must directly follow LINEAR or CONV3X3");
            case PACK_RES_END:
                return fail(PACK_ESHAPE, who + "RES_END must directly follow a CONV3X3");
            default:
                return fail(PACK_EINVAL, who + "unknown op " + std::to_string(L.op));
        }
    }
    if (!res_stack.empty()) return fail(PACK_ESHAPE, who + "RES_BEGIN without RES_END");
    if (m.nodes.empty() || m.nodes.back().kind != NODE_LINEAR || m.nodes.back().act)
        return fail(PACK_ESHAPE, who + "the layer list must end in a LINEAR layer producing the logits");
    m.tensors[cur].f32 = true;
    // The gradient wrt the logits keeps its rows padded to whole 16-byte vectors; the padding is
    // zeroed once at creation and never written, so the classifier's backward products read it
    // with aligned vector loads whatever the number of classes.
    m.tensors[cur].ld_dz = (int)align_up((size_t)m.tensors[cur].c, in.dtype == PACK_BF16 ? 8 : 4);
    m.C = m.tensors[cur].c;
    m.n_params = blob_off;
    // which tensors have parameters upstream
    for (NodeInfo& nd : m.nodes) {
        bool ng = (nd.kind != NODE_GAP) || m.tensors[nd.in_t].needs_grad;
        if (nd.res_src >= 0 && m.tensors[nd.res_src].needs_grad) ng = true;
        m.tensors[nd.out_t].needs_grad = ng;
    }
    return PACK_OK;
}

// ---- plan building ---------------------------------------------------------------------------------
struct DescBuilder {
    std::vector<char> bytes;
    size_t add(const void* p, size_t n) {
        const size_t off = align_up(bytes.size(), 64);
        bytes.resize(off + n);
        if (n) std::memcpy(bytes.data() + off, p, n);
        return off;
    }
};

struct TileOrder { int prob, tm, tn, ks; };

// Hardware deals consecutive workgroup indices round-robin over the 8 XCDs, each with its own L2.
// Logical neighbours (which share an operand tile) are kept together in runs of XCD_RUN tiles on
// one XCD; runs are dealt over the XCDs in rotation so that problems of different cost in one
// launch spread evenly instead of landing on one XCD each.
constexpr size_t XCD_RUN = 8;
// The lean 128 x 64 form (forward, input gradients) hides memory latency by occupancy (four workgroups
// per compute unit) instead of by prefetch depth, so it needs a launch with enough tiles to reach that
// occupancy and a reduction short enough that the prologue and epilogue weigh more than the main loop
// (measured: configs 3 and 5 gain 5 % and 8 % of their step with reductions up to 18 chunks; the
// 256-tile launches of config 2 lose 15 %).
constexpr int LEAN64_MAX_CHUNKS = 18;
constexpr size_t LEAN64_MIN_TILES = 1024;
std::vector<TileRef> xcd_order(const std::vector<TileOrder>& logical) {
    const size_t n = align_up(std::max<size_t>(logical.size(), 1), 8 * XCD_RUN);
    std::vector<TileRef> out(n, TileRef{-1, 0, 0, 0});
    for (size_t t = 0; t < logical.size(); ++t) {
        const size_t run = t / XCD_RUN, in_run = t % XCD_RUN;
        const size_t xcd = run % 8, slot = (run / 8) * XCD_RUN + in_run;
        out[slot * 8 + xcd] = TileRef{logical[t].prob, logical[t].tm, logical[t].tn, logical[t].ks};
    }
    while (out.size() > 8 && std::all_of(out.end() - 8, out.end(), [](const TileRef& r) { return r.prob < 0; }))
        out.resize(out.size() - 8);
    return out;
}

// The other way to deal tiles: by member.  All tiles of a member (of every layer in the launch) go to
// one XCD, so the member's activations and output gradients are fetched into one L2 instead of all
// eight; members are spread over the XCDs so that the XCDs' totals match (largest first, each to the
// least loaded XCD).  With fewer than 8 members each one is cut into 8 / K parts that take every
// P-th column strip of each of its problems.  Every XCD walks its tiles in the launch's slow-first
// problem order, which keeps tiles of like cost at like positions on all eight (workgroups are
// handed out in index order, so an XCD whose next tile is slow may hold back the others).
// Used for the weight gradients of dense layers.  cost[t]: tile t's estimate in arbitrary units.
std::vector<TileRef> xcd_by_member(const std::vector<TileOrder>& logical, const std::vector<double>& cost,
                                   const std::vector<GemmProb>& probs) {
    std::vector<int> ids;
    for (const GemmProb& g : probs)
        if (std::find(ids.begin(), ids.end(), g.member) == ids.end()) ids.push_back(g.member);
    const int parts = std::max(1, 8 / (int)std::max<size_t>(ids.size(), 1));
    auto unit_of = [&](size_t t) {
        const int m = (int)(std::find(ids.begin(), ids.end(), probs[logical[t].prob].member) - ids.begin());
        return m * parts + (logical[t].tn + logical[t].ks) % parts;
    };
    std::vector<double> unit_cost(ids.size() * parts, 0.0);
    for (size_t t = 0; t < logical.size(); ++t) unit_cost[unit_of(t)] += cost[t];
    std::vector<int> order(unit_cost.size());
    for (size_t u = 0; u < order.size(); ++u) order[u] = (int)u;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return unit_cost[x] > unit_cost[y]; });
    std::vector<int> xcd_of(unit_cost.size(), 0);
    double load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int u : order) {
        const int j = (int)(std::min_element(load, load + 8) - load);
        xcd_of[u] = j;
        load[j] += unit_cost[u];
    }
    std::vector<std::vector<TileRef>> per(8);
    for (size_t t = 0; t < logical.size(); ++t)
        per[xcd_of[unit_of(t)]].push_back(TileRef{logical[t].prob, logical[t].tm, logical[t].tn, logical[t].ks});
    size_t longest = 1;
    for (const auto& v : per) longest = std::max(longest, v.size());
    std::vector<TileRef> out(longest * 8, TileRef{-1, 0, 0, 0});
    for (size_t j = 0; j < 8; ++j)
        for (size_t i = 0; i < per[j].size(); ++i) out[i * 8 + j] = per[j][i];
    return out;
}

// rows of the problem are pixels of a w-wide, hw-pixel image plane
void set_row_space(GemmProb& g, int w, int hw) {
    g.row_w = w;
    g.row_hw = hw;
    auto lg = [](int v) { int l = 0; while ((1 << l) < v) ++l; return ((1 << l) == v) ? l : -1; };
    g.lg_row_w = lg(w);
    g.lg_row_hw = lg(hw);
    if (g.lg_row_w < 0 || g.lg_row_hw < 0) g.lg_row_w = g.lg_row_hw = -1;
}

size_t count_tiles(const std::vector<GemmProb>& probs, int cfg) {
    size_t n = 0;
    for (const GemmProb& g : probs) {
        const size_t tms = (g.R + GEMM_TILE_M[cfg] - 1) / GEMM_TILE_M[cfg];
        const size_t tns = (g.Q + GEMM_TILE_N[cfg] - 1) / GEMM_TILE_N[cfg];
        n += tms * tns * std::max(1, (g.Kd + g.ksplit - 1) / g.ksplit);
    }
    return n;
}

double padded_work(const GemmProb& g, int c) {
    const double tms = (g.R + GEMM_TILE_M[c] - 1) / GEMM_TILE_M[c], tns = (g.Q + GEMM_TILE_N[c] - 1) / GEMM_TILE_N[c];
    return tms * GEMM_TILE_M[c] * tns * GEMM_TILE_N[c] * (double)std::min(g.Kd, g.ksplit) *
           std::max(1, (g.Kd + g.ksplit - 1) / g.ksplit);
}

void emit_gemm_launch(pack_ctx* p, DescBuilder& db, int mode, int cfg, const std::vector<GemmProb>& probs) {
    const int BMc = GEMM_TILE_M[cfg], BNc = GEMM_TILE_N[cfg];
    std::vector<TileOrder> logical;
    for (size_t i = 0; i < probs.size(); ++i) {
        const GemmProb& g = probs[i];
        const int tms = (g.R + BMc - 1) / BMc, tns = (g.Q + BNc - 1) / BNc;
        const int S = (g.Kd + g.ksplit - 1) / g.ksplit;
        for (int ks = 0; ks < std::max(S, 1); ++ks) {
            if (mode == CONV_FWD || mode == CONV_DX) {
                for (int tm = 0; tm < tms; ++tm)
                    for (int tn = 0; tn < tns; ++tn) logical.push_back({(int)i, tm, tn, ks});
            } else {
                for (int tn = 0; tn < tns; ++tn)
                    for (int tm = 0; tm < tms; ++tm) logical.push_back({(int)i, tm, tn, ks});
            }
        }
    }
    std::vector<TileRef> tiles;
    // by member only where every XCD then walks the same sequence of tiles: members with identical
    // problem lists, no split reductions, and a member count that divides or is divided by 8
    // (measured: 4 % faster on 8 equal MLPs, 5 % slower on 32 mixed MLPs and several times slower on
    // split reductions, so those keep the rotating deal).  PACK_XCD_ROTATE: measuring aid.
    bool by_member = mode == LIN_DW && !std::getenv("PACK_XCD_ROTATE");
    if (by_member) {
        std::vector<int> ids;
        std::vector<std::vector<long long>> shape;
        for (const GemmProb& g : probs) {
            size_t m = std::find(ids.begin(), ids.end(), g.member) - ids.begin();
            if (m == ids.size()) { ids.push_back(g.member); shape.emplace_back(); }
            shape[m].insert(shape[m].end(), {g.R, g.Q, g.Kd});
            if (g.Kd > g.ksplit) by_member = false;
        }
        for (const auto& sh : shape) by_member = by_member && sh == shape[0];
        by_member = by_member && !ids.empty() && (ids.size() % 8 == 0 || 8 % ids.size() == 0);
    }
    if (by_member) {
        // chunks of the reduction + the epilogue (a tile's weights read and written), in chunk units
        std::vector<double> cost(logical.size());
        for (size_t t = 0; t < logical.size(); ++t) {
            const GemmProb& g = probs[logical[t].prob];
            const int chunk = p->bf16 ? 64 : 32;
            const double rows = std::min(BMc, g.R - logical[t].tm * BMc), cols = std::min(BNc, g.Q - logical[t].tn * BNc);
            cost[t] = 10.0 * rows * cols / ((double)BMc * BNc) + (double)((std::min(g.Kd, g.ksplit) + chunk - 1) / chunk);
        }
        tiles = xcd_by_member(logical, cost, probs);
    } else {
        tiles = xcd_order(logical);
    }
    Launch L;
    L.kind = L_GEMM;
    L.mode = mode;
    L.tile_cfg = cfg;
    L.desc_off = db.add(probs.data(), probs.size() * sizeof(GemmProb));
    L.map_off = db.add(tiles.data(), tiles.size() * sizeof(TileRef));
    L.n = (int)tiles.size();
    const double esz = p->bf16 ? 2.0 : 4.0;
    // An operand that several problems of the launch read (the shared input batch or its im2col copy,
    // Section 3.4) counts once, at the size of its largest reader (smaller batches are prefixes of it).
    std::map<std::pair<int, long long>, double> shared_a, shared_b;
    auto operand_key = [](const void* ptr, bool is_input, long long x_off) {
        return is_input ? std::make_pair(1, x_off) : std::make_pair(0, (long long)(uintptr_t)ptr);
    };
    for (const GemmProb& g : probs) {
        L.flops += 2.0 * g.R * g.Q * g.Kd;
        const double out = (double)g.R * g.Q;
        double a = 0, b = 0, c = 0;
        switch (mode) {
            case LIN_FWD: a = (double)g.R * g.Kd; b = (double)g.Q * g.Kd; c = out * ((g.flags & F_OUT_F32) ? 4.0 : esz) / esz; break;
            case LIN_DX: a = (double)g.R * g.Kd; b = (double)g.Q * g.Kd; c = out * (1.0 + ((g.flags & F_MASK) ? 1.0 : 0.0) + ((g.flags & F_ACCUM) ? 1.0 : 0.0)); break;
            case LIN_DW: a = (double)g.R * g.Kd; b = (double)g.Q * g.Kd; break;
            case CONV_FWD: a = (double)g.R / (g.Ho * g.Wo) * g.H * g.W * g.Cin; b = (double)g.Q * g.Kd; c = out; break;
            case CONV_DX: a = (double)g.R * g.Cout / ((g.flags & F_ROWMAP) ? 1.0 : (double)(g.stride * g.stride)); b = (double)g.Q * g.Kd;
                          c = out * (1.0 + ((g.flags & F_MASK) ? 1.0 : 0.0) + ((g.flags & F_ACCUM) ? 1.0 : 0.0)); break;
            default: a = (double)g.R * g.Kd; b = (double)g.Kd / (g.Ho * g.Wo) * g.H * g.W * g.Cin; break;
        }
        double& sa = shared_a[operand_key(g.A, (g.flags & F_A_INPUT) != 0, g.x_off)];
        double& sb = shared_b[operand_key(g.B, (g.flags & F_B_INPUT) != 0, g.x_off)];
        sa = std::max(sa, a);
        sb = std::max(sb, b);
        L.bytes += c * esz;
        if (mode == LIN_DW || mode == CONV_DW) {
            const double splits = std::max(1, (g.Kd + g.ksplit - 1) / g.ksplit);
            if (!(g.flags & F_UPDATE) || (g.flags & F_KEEP_G)) L.bytes += out * 4.0 * splits;      // gradient (or partials) written
            if (g.flags & F_UPDATE) L.bytes += out * (8.0 + (g.upd_shadow ? 2.0 : 0.0));            // W read + written, bf16 copy written
        }
    }
    for (const auto& kv : shared_a) L.bytes += kv.second * esz;
    for (const auto& kv : shared_b) L.bytes += kv.second * esz;
    p->plan.push_back(L);
}

void add_gemm_launch(pack_ctx* p, DescBuilder& db, int mode, const std::vector<GemmProb>& all_probs_in) {
    // PACK_GENERAL_TAIL: every forward / input-gradient tile takes the general form of the tail, for the test that
    // compares it bit for bit with the form whole tiles of the plain cases take
    std::vector<GemmProb> all_probs = all_probs_in;
    if (std::getenv("PACK_GENERAL_TAIL"))
        for (GemmProb& g : all_probs) g.flags |= F_GENERAL_TAIL;
    // problems whose operands are not aligned for 16-byte loads go to the scalar-gather kernel
    std::vector<GemmProb> probs, scalar;
    for (const GemmProb& g : all_probs) {
        bool vec = (g.flags & F_VEC_A) && (g.flags & F_VEC_B);
        if (vec) {
            // The aligned kernels address an operand with 32-bit byte offsets inside a 2 GB window:
            // larger operands (and weight-gradient convolutions over images narrower than the four
            // pixels a load block covers) take the scalar kernel.
            const double esz = p->bf16 ? 2.0 : 4.0;
            double ea = 0, eb = 0;
            switch (mode) {
                case LIN_FWD: ea = (double)g.R * g.lda; eb = (double)g.Q * g.ldb; break;
                case LIN_DX: ea = (double)g.R * g.lda; eb = (double)g.Kd * g.ldb; break;
                case LIN_DW: ea = (double)g.Kd * g.lda; eb = (double)g.Kd * g.ldb; break;
                case CONV_FWD: ea = (double)g.R / (g.Ho * g.Wo) * g.H * g.W * g.Cin + (g.W + 1) * g.Cin; eb = (double)g.Q * g.ldb; break;
                case CONV_DX: {
                    const double images = (double)g.R / ((g.flags & F_ROWMAP) ? g.cls_h * g.cls_w : g.H * g.W);
                    ea = images * g.Ho * g.Wo * g.Cout + (g.Wo + 1) * g.Cout;
                    eb = (double)g.Q * g.ldb;
                    break;
                }
                default:
                    ea = (double)g.Kd * g.lda;
                    eb = (double)g.Kd / (g.Ho * g.Wo) * g.H * g.W * g.Cin + (g.W + 1) * g.Cin;
                    if (g.Wo < 4) vec = false;
                    break;
            }
            if (ea * esz >= 2.0e9 || eb * esz >= 2.0e9) vec = false;
            if ((g.flags & (F_A_INPUT | F_B_INPUT | F_AUX_INPUT)) && (g.x_off & 15)) vec = false;
        }
        if (vec) {
            probs.push_back(g);
        } else {
            GemmProb gs = g;
            gs.flags &= ~(F_VEC_A | F_VEC_B);
            scalar.push_back(gs);
        }
    }
    if (!scalar.empty()) emit_gemm_launch(p, db, mode, GEMM_CFG_SCALAR, scalar);
    if (mode == CONV_DW && !std::getenv("PACK_NO_HALO_DW")) {
        // convolution weight gradients whose shape allows it take the halo form (all nine taps of a block of
        // channel pairs in one workgroup; the input staged once per chunk of pixels): one launch per stride.
        // PACK_NO_HALO_DW keeps them on the staged-tile form, for the test that compares the two bit for bit.
        std::vector<GemmProb> halo[3], rest;
        for (const GemmProb& g : probs) {
            const int cfg = conv_dw_halo_cfg(p->bf16, g);
            if (cfg >= 0) halo[cfg - GEMM_CFG_HALO_S1].push_back(g);
            else rest.push_back(g);
        }
        for (int c = 0; c < 3; ++c)
            if (!halo[c].empty()) emit_gemm_launch(p, db, mode, GEMM_CFG_HALO_S1 + c, halo[c]);
        probs.swap(rest);
    }
    if ((mode == CONV_FWD || mode == CONV_DX) && !std::getenv("PACK_NO_HALO_ROWS")) {
        // stride-1 convolutions whose shape allows it take the halo form of the forward pass and input gradient
        // (the pixels a tile's taps reach staged once per block of channels).  Whether a problem does depends on
        // its own shape only, so a member's bits do not depend on who else is in the pack.
        // PACK_NO_HALO_ROWS keeps them on the staged-tile form, for the test that compares the two.
        std::vector<GemmProb> rows[2], rest;
        for (const GemmProb& g : probs) {
            const int cfg = conv_rows_halo_cfg(p->bf16, mode, g);
            if (cfg >= 0) rows[cfg - GEMM_CFG_ROWS64].push_back(g);
            else rest.push_back(g);
        }
        for (int c = 0; c < 2; ++c)
            if (!rows[c].empty()) emit_gemm_launch(p, db, mode, GEMM_CFG_ROWS64 + c, rows[c]);
        probs.swap(rest);
    }
    if (probs.empty()) return;
    // The tile shape only partitions the output; the summation order of an element does not
    // depend on it, so a member's bits do not depend on who else is in the launch.  Each problem
    // prefers the shape that multiplies the fewest padding elements (a 64-channel layer wastes
    // half of a 128-wide tile); the launch as a whole needs enough workgroups to fill the 256
    // compute units about twice.  Problems whose preferred shape carries little of the work
    // ride along in the main launch rather than paying for a launch of their own.
    // (measured: dense products are better off with one larger tile per compute unit than with two
    // smaller ones, convolutions the other way round)
    size_t min_tiles = (mode == LIN_FWD || mode == LIN_DX || mode == LIN_DW) ? 256 : 512;
    if (const char* v = std::getenv("PACK_MIN_TILES")) min_tiles = (size_t)std::max(1, std::atoi(v));   // tests: large-pack tile shapes on small cases
    int floor_cfg = 0;
    while (floor_cfg < 2 && count_tiles(probs, floor_cfg) < min_tiles) ++floor_cfg;
    std::vector<int> want(probs.size());
    double work[3] = {0, 0, 0}, total = 0;
    for (size_t i = 0; i < probs.size(); ++i) {
        int c = floor_cfg;
        while (c < 2 && padded_work(probs[i], c + 1) < 0.8 * padded_work(probs[i], c)) ++c;
        want[i] = c;
        work[c] += padded_work(probs[i], c);
        total += padded_work(probs[i], c);
    }
    int main_cfg = 0;
    for (int c = 1; c < 3; ++c)
        if (work[c] > work[main_cfg]) main_cfg = c;
    // weight gradients whose reduction is at most a few chunks long take the lean form of the
    // 128 x 128 kernel (more tiles resident per compute unit)
    const bool lean_ok = (mode == LIN_DW || mode == CONV_DW);
    // forward products and input gradients on 128 x 64 tiles have a lean form too (one register stage,
    // one operand buffer, four workgroups per compute unit); PACK_LEAN64_CHUNKS sets the longest
    // reduction, in chunks, that takes it (0: never; a measuring aid)
    int lean64_chunks = LEAN64_MAX_CHUNKS;
    if (const char* v = std::getenv("PACK_LEAN64_CHUNKS")) lean64_chunks = std::atoi(v);
    const bool is_dw = mode == LIN_DW || mode == CONV_DW;
    const int chunk_k = p->bf16 ? 64 : 32;
    for (int c = 0; c < 3; ++c) {
        std::vector<GemmProb> group, lean;
        for (size_t i = 0; i < probs.size(); ++i) {
            const int eff = (work[want[i]] < 0.15 * total) ? main_cfg : want[i];
            if (eff != c) continue;
            const int chunks = (std::min(probs[i].Kd, probs[i].ksplit) + chunk_k - 1) / chunk_k;
            if (c == 0 && lean_ok && chunks <= 8) lean.push_back(probs[i]);
            else if (c == 1 && !is_dw && chunks <= lean64_chunks) lean.push_back(probs[i]);
            else group.push_back(probs[i]);
        }
        if (!is_dw && !lean.empty() && count_tiles(lean, GEMM_CFG_LEAN64) < LEAN64_MIN_TILES && !std::getenv("PACK_LEAN64_CHUNKS")) {
            group.insert(group.end(), lean.begin(), lean.end());   // too few tiles to fill the occupancy
            lean.clear();
        }
        if (!lean.empty()) emit_gemm_launch(p, db, mode, is_dw ? GEMM_CFG_LEAN : GEMM_CFG_LEAN64, lean);
        if (!group.empty()) emit_gemm_launch(p, db, mode, c, group);
    }
}

template <typename P>
void add_mapped_launch(pack_ctx* p, DescBuilder& db, int kind, const std::vector<P>& probs,
                       const std::vector<int>& blocks_per_prob) {
    if (probs.empty()) return;
    std::vector<int2> map;
    for (size_t i = 0; i < probs.size(); ++i)
        for (int b = 0; b < blocks_per_prob[i]; ++b) map.push_back(int2{(int)i, b});
    if (map.empty()) return;
    Launch L;
    L.kind = kind;
    L.desc_off = db.add(probs.data(), probs.size() * sizeof(P));
    L.map_off = db.add(map.data(), map.size() * sizeof(int2));
    L.n = (int)map.size();
    p->plan.push_back(L);
}

inline int elem_vec(bool bf16) { return bf16 ? 8 : 4; }

// the gather kernels index with 32-bit element offsets
inline bool small_tensors(const TensorInfo& a, const TensorInfo& b) {
    return a.elems() < (size_t)1 << 30 && b.elems() < (size_t)1 << 30;
}

// Builds the whole launch sequence.  Workspace offsets are relative; `ws_need` returns the size.
void build_plan(pack_ctx* p, DescBuilder& db, size_t& ws_need) {
    const bool bf = p->bf16;
    const int V = elem_vec(bf);
    const int BKc = bf ? 64 : 32;   // reduction indices per LDS chunk (ET<T>::BK of the kernels)
    const size_t esz = bf ? 2 : 4;
    size_t max_nodes = 0;
    for (const ModelInfo& m : p->models) max_nodes = std::max(max_nodes, m.nodes.size());
    ws_need = 0;

    const long long block_bytes = (long long)p->in.B * p->in.in_h * p->in.in_w * p->in.in_c * (long long)esz;
    auto x_off = [&](const ModelInfo& m) -> long long {
        return p->own_input ? (long long)(&m - p->models.data()) * block_bytes : 0;
    };
    auto weight_ptr = [&](const NodeInfo& nd) -> const void* {
        return bf ? (const void*)((const char*)p->shadow + nd.w_off * 2) : (const void*)(p->master + nd.w_off);
    };

    // ---------------- shared-input loader ----------------
    for (size_t i = 0; i < p->im2col.size(); ++i) {
        Launch L;
        L.kind = L_IM2COL;
        L.mode = (int)i;
        L.n = 1;
        p->plan.push_back(L);
    }

    // ---------------- forward ----------------
    for (size_t s = 0; s < max_nodes; ++s) {
        std::vector<GemmProb> lin, conv;
        std::vector<GapProb> gaps;
        std::vector<int> gap_blocks;
        for (ModelInfo& m : p->models) {
            if (s >= m.nodes.size()) continue;
            const NodeInfo& nd = m.nodes[s];
            const TensorInfo& ti = m.tensors[nd.in_t];
            const TensorInfo& to = m.tensors[nd.out_t];
            if (nd.kind == NODE_GAP) {
                GapProb g{};
                g.in = ti.act; g.out = to.act; g.n = ti.n; g.hw = ti.h * ti.w; g.c = ti.c;
                gaps.push_back(g);
                gap_blocks.push_back((ti.n * ti.c + 255) / 256);
                continue;
            }
            if (m.fused_head && s + 1 == m.nodes.size()) continue;   // part of the head kernel
            GemmProb g{};
            g.zeros = p->zeros;
            g.x_off = x_off(m);
            g.A = ti.is_input ? nullptr : ti.act;
            g.B = weight_ptr(nd);
            g.C = to.act;
            g.bias = p->master + nd.b_off;
            g.flags = (nd.act == ACT_RELU ? F_RELU : 0) | (to.f32 ? F_OUT_F32 : 0) | (ti.is_input ? F_A_INPUT : 0);
            g.act = nd.act;
            if (nd.kind == NODE_LINEAR) {
                g.R = ti.n; g.Q = nd.out; g.Kd = nd.fan_in;
                g.lda = nd.fan_in; g.ldb = nd.fan_in; g.ldc = nd.out;
                if (g.Kd % V == 0) g.flags |= F_VEC_A | F_VEC_B;
                g.ksplit = g.Kd;
                lin.push_back(g);
            } else if (nd.kp) {
                // first convolution over the shared im2col buffer: a dense product, rows = pixels
                g.A = p->im2col[nd.im2col_idx].out;
                g.flags &= ~F_A_INPUT;
                g.H = ti.h; g.W = ti.w; g.Cin = ti.c; g.Ho = to.h; g.Wo = to.w; g.Cout = to.c; g.stride = nd.stride;
                g.R = to.n * to.h * to.w; g.Q = to.c; g.Kd = nd.kp;
                set_row_space(g, to.w, to.h * to.w);
                g.lda = nd.kp; g.ldb = nd.kp; g.ldc = to.c;
                g.flags |= F_VEC_A | F_VEC_B;
                if (nd.res_src >= 0) {
                    const TensorInfo& rs = m.tensors[nd.res_src];
                    g.aux = rs.is_input ? nullptr : rs.act;
                    if (rs.is_input) g.flags |= F_AUX_INPUT;
                    g.flags |= nd.res_down ? F_RES_DOWN : F_RES_ID;
                    g.resH = rs.h; g.resW = rs.w; g.resC = rs.c;
                }
                g.ksplit = g.Kd;
                lin.push_back(g);
            } else {
                g.H = ti.h; g.W = ti.w; g.Cin = ti.c; g.Ho = to.h; g.Wo = to.w; g.Cout = to.c; g.stride = nd.stride;
                g.R = to.n * to.h * to.w; g.Q = to.c; g.Kd = 9 * ti.c;
                set_row_space(g, to.w, to.h * to.w);
                g.lda = ti.c; g.ldb = 9 * ti.c; g.ldc = to.c;
                // vector path of the gathered operand: a chunk must stay inside one tap
                if (ti.c % BKc == 0 && small_tensors(ti, to)) g.flags |= F_VEC_A | F_VEC_B;
                if (nd.res_src >= 0) {
                    const TensorInfo& rs = m.tensors[nd.res_src];
                    g.aux = rs.is_input ? nullptr : rs.act;
                    if (rs.is_input) g.flags |= F_AUX_INPUT;
                    g.flags |= nd.res_down ? F_RES_DOWN : F_RES_ID;
                    g.resH = rs.h; g.resW = rs.w; g.resC = rs.c;
                }
                g.ksplit = g.Kd;
                conv.push_back(g);
            }
        }
        add_gemm_launch(p, db, LIN_FWD, lin);
        add_gemm_launch(p, db, CONV_FWD, conv);
        add_mapped_launch(p, db, L_GAP_FWD, gaps, gap_blocks);
    }

    // ---------------- loss ----------------
    {
        std::vector<CeProb> ce;
        std::vector<HeadProb> heads;
        std::vector<int> head_blocks;
        for (ModelInfo& m : p->models) {
            if (m.vacant) continue;
            const TensorInfo& lg = m.tensors[m.nodes.back().out_t];
            if (m.fused_head) {
                const NodeInfo& nd = m.nodes.back();
                const TensorInfo& ti = m.tensors[nd.in_t];
                HeadProb h{};
                h.h = ti.act; h.W = weight_ptr(nd); h.bias = p->master + nd.b_off;
                h.logits = (float*)lg.act; h.dlogits = lg.dz; h.dh = ti.needs_grad ? ti.dz : nullptr;
                h.pred = m.pred; h.loss = m.loss; h.partial = m.head_partial;
                h.rows = m.batch; h.C = m.C; h.Kd = nd.fan_in; h.ldd = lg.ld_dz;
                h.label_off = p->own_input ? (int)(&m - p->models.data()) * p->in.B : 0;
                h.mask_act = ti.act_out;
                h.nblk = (m.batch + HEAD_ROWS - 1) / HEAD_ROWS;
                heads.push_back(h);
                head_blocks.push_back(h.nblk);
                continue;
            }
            CeProb c{};
            c.logits = (const float*)lg.act; c.dlogits = lg.dz; c.pred = m.pred; c.loss = m.loss;
            c.rows = m.batch; c.C = m.C; c.ld = m.C; c.ldd = lg.ld_dz;
            c.label_off = p->own_input ? (int)(&m - p->models.data()) * p->in.B : 0;
            ce.push_back(c);
        }
        if (!ce.empty()) {
            Launch L;
            L.kind = L_CE;
            L.desc_off = db.add(ce.data(), ce.size() * sizeof(CeProb));
            L.n = (int)ce.size();
            p->plan.push_back(L);
        }
        add_mapped_launch(p, db, L_HEAD, heads, head_blocks);
        p->n_heads = (int)heads.size();
        if (!heads.empty()) {
            p->head_desc_off = p->plan.back().desc_off;
            for (const HeadProb& h : heads) p->plan.back().mode = std::max(p->plan.back().mode, h.C);   // largest class count
        }
    }

    // ---------------- backward ----------------
    for (ModelInfo& m : p->models)
        for (TensorInfo& t : m.tensors) {
            t.grad_written = false;
            t.sc_dz = nullptr;
        }
    // Weight gradients need only dz and the stored activations, not each other, so all of them
    // run in ONE launch (per kernel kind) after the chain of input gradients: the small layers
    // fill the gaps the big ones leave instead of each paying a launch of its own.
    {
        std::vector<TransposeProb> tps;
        std::vector<int> tp_blocks;
        for (ModelInfo& m : p->models)
            for (const NodeInfo& nd : m.nodes) {
                if (!nd.has_wt) continue;
                TransposeProb t{};
                t.src = weight_ptr(nd);
                t.dst = (char*)p->wt + nd.wt_off * esz;
                t.Cin = m.tensors[nd.in_t].c; t.Cout = nd.out;
                t.tiles_ci = (t.Cin + 63) / 64; t.tiles_co = (t.Cout + 63) / 64;
                tps.push_back(t);
                tp_blocks.push_back(9 * t.tiles_ci * t.tiles_co);
            }
        add_mapped_launch(p, db, L_WTRANS, tps, tp_blocks);
    }
    std::vector<ReduceProb> dw_red;
    std::vector<int> dw_red_blocks;
    std::vector<GemmProb> lin_dw, conv_dw;
    size_t ws_off = 0;
    for (size_t s = max_nodes; s-- > 0;) {
        std::vector<GemmProb> lin_dx, conv_dx;
        std::vector<GapProb> gaps;
        std::vector<int> gap_blocks;
        std::vector<ShortcutProb> scs;
        std::vector<int> sc_blocks;
        for (ModelInfo& m : p->models) {
            if (s >= m.nodes.size()) continue;
            const NodeInfo& nd = m.nodes[s];
            TensorInfo& ti = m.tensors[nd.in_t];
            const TensorInfo& to = m.tensors[nd.out_t];
            if (nd.kind == NODE_GAP) {
                if (!ti.needs_grad) continue;
                GapProb g{};
                g.in = ti.act; g.dz_out = to.dz; g.dz_in = ti.dz; g.n = ti.n; g.hw = ti.h * ti.w; g.c = ti.c;
                g.mask = ti.act_out; g.accum = ti.grad_written;
                ti.grad_written = true;
                gaps.push_back(g);
                gap_blocks.push_back((int)((ti.elems() + ELEMWISE_PER_BLOCK - 1) / ELEMWISE_PER_BLOCK));
                continue;
            }
            const int rows = (nd.kind == NODE_LINEAR) ? to.n : to.n * to.h * to.w;
            // weight gradient
            {
                GemmProb g{};
                g.zeros = p->zeros;
                g.x_off = x_off(m);
                g.A = to.dz;
                g.B = ti.is_input ? nullptr : ti.act;
                g.flags = ti.is_input ? F_B_INPUT : 0;
                const int q_dim = nd.kp ? nd.kp : nd.fan_in;   // columns of the weight matrix in the arena
                g.R = nd.out; g.Q = q_dim; g.Kd = rows;
                g.lda = to.ld_dz ? to.ld_dz : nd.out; g.ldc = q_dim;
                if (g.lda % V == 0) g.flags |= F_VEC_A;
                float* dst = p->grad + nd.w_off;
                const bool dense = (nd.kind == NODE_LINEAR) || nd.kp;
                if (dense) {
                    g.ldb = q_dim;
                    if (nd.kp) {
                        g.B = p->im2col[nd.im2col_idx].out;
                        g.flags &= ~F_B_INPUT;
                    }
                    if (q_dim % V == 0) g.flags |= F_VEC_B;
                } else {
                    g.H = ti.h; g.W = ti.w; g.Cin = ti.c; g.Ho = to.h; g.Wo = to.w; g.Cout = to.c; g.stride = nd.stride;
                    g.ldb = ti.c;
                    // vector path of the gathered input: chunks of output pixels must stay inside
                    // one image and rows must decode by shifts
                    const bool pow2 = (to.w & (to.w - 1)) == 0;
                    if (ti.c % V == 0 && pow2 && (to.h * to.w) % BKc == 0 && small_tensors(ti, to)) g.flags |= F_VEC_B;
                    else g.flags &= ~F_VEC_A;
                }
                // long reductions (many pixels) are split over workgroups; the split length
                // depends on the layer shape only, partial results are summed in split order
                int S;
                if (dense) {
                    const int out_tiles = ((nd.out + 127) / 128) * ((q_dim + 127) / 128);
                    const int chunk = (out_tiles == 1) ? 1024 : 8192;   // a one-tile output gets its parallelism from splits
                    S = std::min(128, std::max(1, (rows + chunk - 1) / chunk));
                } else {
                    // Convolutions: a split is sized for some tens of microseconds of matrix work per
                    // workgroup (the float matrix rate is a sixteenth of the bfloat16 one), and a layer
                    // with few channel blocks is split further until it offers at least 32 workgroups.
                    // Only the layer's own shape enters, so a member's split does not depend on its pack.
                    const int target = bf ? 8192 : 1024;
                    S = std::min(128, std::max(1, (rows + target - 1) / target));
                    const int blocks = ((nd.out + 63) / 64) * ((ti.c + 63) / 64);
                    while (S < 128 && S * blocks < 32 && rows / (2 * S) >= 8 * BKc) S *= 2;
                }
                g.ksplit = (int)align_up((size_t)(rows + S - 1) / S, 64);
                S = (rows + g.ksplit - 1) / g.ksplit;
                const int member = (int)(&m - p->models.data());
                void* const shadow_w = bf ? (void*)((char*)p->shadow + nd.w_off * 2) : nullptr;
                if (S > 1) {
                    // partial sums live in the step's workspace, addressed by offset: the kernels receive the
                    // workspace as an argument (the pack's own, or the library's static scratch array)
                    g.flags |= F_WS;
                    g.C = (void*)(uintptr_t)ws_off;
                    g.split_stride = (long long)nd.w_arena;
                    ReduceProb r{};
                    r.in = (const float*)(uintptr_t)ws_off; r.out = dst; r.stride = (long long)nd.w_arena; r.n = (int)nd.w_arena; r.S = S;
                    if (p->fused) { r.upd_w = p->master + nd.w_off; r.upd_shadow = shadow_w; r.member = member; r.keep_g = p->keep_grads; }
                    dw_red.push_back(r);
                    dw_red_blocks.push_back((int)((nd.w_arena + 1023) / 1024));
                    ws_off += align_up((size_t)S * nd.w_arena * 4, 256);
                    g.dbias = (float*)(uintptr_t)ws_off;
                    ReduceProb rb{};
                    rb.in = (const float*)(uintptr_t)ws_off; rb.out = p->grad + nd.b_off; rb.stride = nd.out; rb.n = nd.out; rb.S = S;
                    if (p->fused) { rb.upd_w = p->master + nd.b_off; rb.member = member; rb.keep_g = p->keep_grads; }
                    dw_red.push_back(rb);
                    dw_red_blocks.push_back((nd.out + 1023) / 1024);
                    ws_off += align_up((size_t)S * nd.out * 4, 256);
                } else {
                    g.ksplit = std::max(g.Kd, 1);
                    g.C = dst;
                    g.dbias = p->grad + nd.b_off;
                    if (p->fused) {
                        g.flags |= F_UPDATE | (p->keep_grads ? F_KEEP_G : 0);
                        g.upd_w = p->master + nd.w_off; g.upd_shadow = shadow_w; g.upd_b = p->master + nd.b_off; g.member = member;
                    }
                }
                if (dense) lin_dw.push_back(g);
                else conv_dw.push_back(g);
            }
            // input gradient (the head kernel has already written it for a fused classifier head)
            if (m.fused_head && s + 1 == m.nodes.size()) {
                if (ti.needs_grad) ti.grad_written = true;
            } else if (ti.needs_grad) {
                GemmProb g{};
                g.zeros = p->zeros;
                g.A = to.dz;
                g.B = weight_ptr(nd);
                g.C = ti.dz;
                g.aux = ti.act;
                g.flags = (ti.act_out ? F_MASK : 0) | (ti.grad_written ? F_ACCUM : 0);
                g.mask_act = ti.act_out;
                ti.grad_written = true;
                if (nd.kind == NODE_LINEAR) {
                    g.R = ti.n; g.Q = nd.fan_in; g.Kd = nd.out;
                    g.lda = to.ld_dz ? to.ld_dz : nd.out; g.ldb = nd.fan_in; g.ldc = nd.fan_in;
                    if (g.lda % V == 0) g.flags |= F_VEC_A;
                    if (nd.fan_in % V == 0) g.flags |= F_VEC_B;
                    g.ksplit = g.Kd;
                    lin_dx.push_back(g);
                } else {
                    g.H = ti.h; g.W = ti.w; g.Cin = ti.c; g.Ho = to.h; g.Wo = to.w; g.Cout = to.c; g.stride = nd.stride;
                    g.R = ti.n * ti.h * ti.w; g.Q = ti.c; g.Kd = 9 * to.c;
                    set_row_space(g, ti.w, ti.h * ti.w);
                    g.B = (const char*)p->wt + nd.wt_off * esz;   // transposed copy [Cin][9][Cout]
                    g.lda = to.c; g.ldb = 9 * to.c; g.ldc = ti.c;
                    if (to.c % BKc == 0 && ti.c % V == 0 && small_tensors(ti, to)) g.flags |= F_VEC_A | F_VEC_B;
                    g.ksplit = g.Kd;
                    const bool with_sc = ti.sc_dz != nullptr;
                    if (with_sc) {
                        g.sc = ti.sc_dz; g.scH = ti.sc_h; g.scW = ti.sc_w; g.scC = ti.sc_c;
                        ti.sc_dz = nullptr;
                    }
                    const int sc_flag = !with_sc ? 0 : (ti.sc_down ? F_SC_DOWN : F_SC_ID);
                    if (nd.stride == 2 && (g.flags & F_VEC_A)) {
                        // An input pixel of a stride-2 convolution receives gradient through the
                        // taps whose parity matches its own only (1, 2, 2 or 4 of the 9): one
                        // problem per parity class multiplies no structural zeros.  The surviving
                        // products are added in the same order as in the undivided sum.
                        for (int py = 0; py < 2; ++py)
                            for (int px = 0; px < 2; ++px) {
                                GemmProb c = g;
                                c.flags |= F_ROWMAP;
                                c.cls_py = py; c.cls_px = px;
                                c.cls_h = py ? (ti.h + 1) / 2 : ti.h / 2;
                                c.cls_w = px ? (ti.w + 1) / 2 : ti.w / 2;
                                c.R = ti.n * c.cls_h * c.cls_w;
                                set_row_space(c, c.cls_w, c.cls_h * c.cls_w);
                                c.Kd = (py ? 1 : 2) * (px ? 1 : 2) * to.c;
                                c.ksplit = c.Kd;
                                if (py && px) c.flags |= sc_flag;   // pixels with even coordinates: the subsampling shortcut's
                                if (c.R > 0) conv_dx.push_back(c);
                            }
                    } else {
                        g.flags |= sc_flag;
                        conv_dx.push_back(g);
                    }
                }
            }
            // gradient through the shortcut into the block input
            if (nd.res_src >= 0 && m.tensors[nd.res_src].needs_grad) {
                TensorInfo& rs = m.tensors[nd.res_src];
                // The block's first layer, if it is a convolution with an input gradient of its own,
                // adds the shortcut's share in its epilogue (it is planned after this node and is
                // then the first writer of the tensor); PACK_NO_FUSED_SHORTCUT is a measuring aid.
                int first = -1, readers = 0;
                for (size_t j = 0; j < m.nodes.size(); ++j)
                    if (m.nodes[j].in_t == nd.res_src) { first = (int)j; ++readers; }
                const bool fuse = readers == 1 && first >= 0 && first < (int)s && m.nodes[first].kind == NODE_CONV && !m.nodes[first].kp && !rs.grad_written &&
                                  !rs.is_input && !(nd.res_down && m.nodes[first].stride != 2) && !std::getenv("PACK_NO_FUSED_SHORTCUT");
                if (fuse) {
                    rs.sc_dz = to.dz; rs.sc_h = to.h; rs.sc_w = to.w; rs.sc_c = to.c; rs.sc_down = nd.res_down;
                    continue;
                }
                ShortcutProb sp{};
                sp.dz_out = to.dz; sp.src = rs.act; sp.dz_src = rs.dz;
                sp.n = rs.n; sp.H = rs.h; sp.W = rs.w; sp.C = rs.c; sp.Ho = to.h; sp.Wo = to.w; sp.Co = to.c;
                sp.down = nd.res_down; sp.mask = rs.act_out; sp.accum = rs.grad_written;
                rs.grad_written = true;
                scs.push_back(sp);
                sc_blocks.push_back((int)((rs.elems() + ELEMWISE_PER_BLOCK - 1) / ELEMWISE_PER_BLOCK));
            }
        }
        add_gemm_launch(p, db, LIN_DX, lin_dx);
        add_gemm_launch(p, db, CONV_DX, conv_dx);
        add_mapped_launch(p, db, L_SHORTCUT, scs, sc_blocks);
        add_mapped_launch(p, db, L_GAP_BWD, gaps, gap_blocks);
    }
    ws_need = ws_off;
    // a grid drains best when its slowest tiles start first: unaligned problems (scalar gather),
    // then long reductions, then large outputs
    auto slow_first = [](const GemmProb& a, const GemmProb& b) {
        const bool va = (a.flags & F_VEC_A) && (a.flags & F_VEC_B), vb = (b.flags & F_VEC_A) && (b.flags & F_VEC_B);
        if (va != vb) return !va;
        if (a.ksplit != b.ksplit) return std::min(a.ksplit, a.Kd) > std::min(b.ksplit, b.Kd);
        return (long long)a.R * a.Q > (long long)b.R * b.Q;
    };
    std::stable_sort(lin_dw.begin(), lin_dw.end(), slow_first);
    std::stable_sort(conv_dw.begin(), conv_dw.end(), slow_first);
    add_gemm_launch(p, db, LIN_DW, lin_dw);
    add_gemm_launch(p, db, CONV_DW, conv_dw);
    add_mapped_launch(p, db, L_REDUCE, dw_red, dw_red_blocks);

    // ---------------- update ----------------
    // (plain-SGD packs have applied it in the weight-gradient launches above)
    if (p->arena_elems && !p->fused) {
        Launch L;
        L.kind = L_SGD;
        L.n = 1;
        p->plan.push_back(L);
    }
}

// frees every device buffer and event the pack holds; the host-side description stays
void free_device(pack_ctx* p) {
    if (p->dry) {
        p->master = p->grad = nullptr; p->shadow = p->wt = nullptr; p->opt_m = p->opt_v = nullptr; p->opt_params = nullptr;
        p->seg_end = nullptr; p->slab = p->workspace = p->desc = nullptr;
        p->dry_regions.clear();
        p->device_bytes = 0;
        return;
    }
    void** bufs[] = {(void**)&p->master, (void**)&p->grad, &p->shadow, &p->wt, (void**)&p->opt_m, (void**)&p->opt_v,
                     (void**)&p->opt_params, (void**)&p->seg_end, (void**)&p->slab, (void**)&p->workspace, (void**)&p->desc};
    for (void** b : bufs) {
        if (*b) (void)hipFree(*b);
        *b = nullptr;
    }
    for (auto& s : p->stamps) { (void)hipEventDestroy(s.t0); (void)hipEventDestroy(s.t1); }
    p->stamps.clear();
    p->profiling = false;
    p->device_bytes = 0;
}

void release(pack_ctx* p) {
    if (!p) return;
    free_device(p);
    delete p;
}

pack_status dev_alloc(void** ptr, size_t bytes, pack_ctx* p) {
    bytes = align_up(std::max<size_t>(bytes, 256), 256);
    if (p->dry) {
        *ptr = (void*)p->dry_next;
        p->dry_regions.push_back({p->dry_next, bytes});
        p->dry_next += align_up(bytes, (size_t)1 << 21) + ((size_t)1 << 21);   // a gap after every allocation
        p->device_bytes += bytes;
        return PACK_OK;
    }
    hipError_t e = hipMalloc(ptr, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *ptr = nullptr;
        return fail(e == hipErrorOutOfMemory ? PACK_ENOMEM : PACK_EDEVICE,
                    std::string("hipMalloc of ") + std::to_string(bytes) + " bytes: " + hipGetErrorString(e));
    }
    p->device_bytes += bytes;
    return PACK_OK;
}

pack_status live_member(const pack_ctx* p, int32_t k);

pack_status upload_weights(pack_ctx* p, int k, const float* blob) {
    ModelInfo& m = p->models[k];
    std::vector<float> arena;
    blob_to_arena(m, blob, arena);
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    HIP_TRY(hipMemcpy(p->master + m.arena_begin, arena.data(), arena.size() * sizeof(float), hipMemcpyHostToDevice), PACK_EDEVICE);
    if (p->bf16) {
        HIP_TRY(launch_cast_bf16(p->master + m.arena_begin, (char*)p->shadow + m.arena_begin * 2,
                                 (long long)arena.size(), p->stream), PACK_EDEVICE);
        HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    }
    return PACK_OK;
}

pack_status download(pack_ctx* p, int k, const float* dev_arena, float* host_dst, size_t n_floats) {
    if (!p || !host_dst) return fail(PACK_EINVAL, "null argument");
    pack_status st = live_member(p, k);
    if (st != PACK_OK) return st;
    ModelInfo& m = p->models[k];
    if (n_floats != m.n_params) return fail(PACK_EINVAL, "n_floats does not match pack_num_params");
    std::vector<float> arena(m.arena_end - m.arena_begin);
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    HIP_TRY(hipMemcpy(arena.data(), dev_arena + m.arena_begin, arena.size() * sizeof(float), hipMemcpyDeviceToHost), PACK_EDEVICE);
    arena_to_blob(m, arena, host_dst);
    return PACK_OK;
}

// Lays the members of p->models out in the parameter arena, allocates every device buffer, builds the
// launch plan and uploads it.  Expects a pack without device buffers; on failure it has none again.
// Weights and optimiser state are zero afterwards (Adagrad accumulators excepted): the caller writes them.
pack_status build_device(pack_ctx* p) {
    const int K = p->K;
    const pack_input_spec* input = &p->in;
    p->im2col.clear();
    p->plan.clear();
    // parameter arena: members back to back, every tensor starting on a 64-element boundary
    size_t off = 0;
    for (ModelInfo& m : p->models) {
        m.arena_begin = off;
        for (NodeInfo& nd : m.nodes) {
            if (nd.kind == NODE_GAP) continue;
            nd.w_off = off;
            off = align_up(off + nd.w_arena, 64);
            nd.b_off = off;
            off = align_up(off + (size_t)nd.out, 64);
        }
        m.arena_end = off;
    }
    p->arena_elems = off;
    const size_t esz = p->bf16 ? 2 : 4;

    pack_status s;
#define TRY_ALLOC(ptr, bytes)                                         \
    if ((s = dev_alloc((void**)&(ptr), (bytes), p)) != PACK_OK) {     \
        free_device(p);                                               \
        return s;                                                     \
    }
    TRY_ALLOC(p->master, p->arena_elems * 4);
    TRY_ALLOC(p->grad, p->arena_elems * 4);
    if (p->bf16) TRY_ALLOC(p->shadow, p->arena_elems * 2);
    TRY_ALLOC(p->seg_end, (size_t)K * sizeof(long long));
    bool need_m = false, need_v = false;
    for (const pack_opt_spec& o : p->opt) {
        if (o.kind != PACK_OPT_SGD) need_m = true;
        if (o.kind == PACK_OPT_ADAM) need_v = true;
    }
    p->any_opt = need_m;
    p->fused = !need_m && !std::getenv("PACK_NO_FUSED_UPDATE");   // the variable is a measuring aid
    if (need_m) {
        TRY_ALLOC(p->opt_m, p->arena_elems * 4);
        TRY_ALLOC(p->opt_params, (size_t)K * sizeof(OptStatic));
    }
    if (need_v) TRY_ALLOC(p->opt_v, p->arena_elems * 4);
    {
        size_t wt_elems = 0;
        for (ModelInfo& m : p->models)
            for (NodeInfo& nd : m.nodes) {
                if (nd.kind != NODE_CONV || nd.kp || !m.tensors[nd.in_t].needs_grad) continue;
                nd.has_wt = true;
                nd.wt_off = wt_elems;
                wt_elems = align_up(wt_elems + nd.w_elems, 64);
            }
        if (wt_elems) TRY_ALLOC(p->wt, wt_elems * esz);
    }

    // one slab for activations, their gradients, predictions, losses and the label-error flag
    size_t slab = 0;
    auto reserve = [&](size_t bytes) { const size_t o = slab; slab += align_up(std::max<size_t>(bytes, 16), 256); return o; };
    std::vector<std::pair<void**, size_t>> fix;
    // shared im2col buffers: one per stride used by a first-layer convolution over few channels
    p->im2col_xoff.clear();
    for (ModelInfo& m : p->models) {
        if (m.vacant) continue;
        NodeInfo& nd = m.nodes[0];
        if (!nd.kp) continue;
        nd.im2col_idx = -1;
        if (!p->own_input)   // one shared input: members with the same first-layer stride share one loader
            for (size_t i = 0; i < p->im2col.size(); ++i)
                if (p->im2col[i].stride == nd.stride) nd.im2col_idx = (int)i;
        if (nd.im2col_idx < 0) {
            Im2colProb ip{};
            ip.B = p->own_input ? m.batch : input->B;
            ip.H = input->in_h; ip.W = input->in_w; ip.C = input->in_c;
            ip.stride = nd.stride; ip.Kp = nd.kp;
            ip.Ho = (ip.H - 1) / nd.stride + 1; ip.Wo = (ip.W - 1) / nd.stride + 1;
            p->im2col.push_back(ip);
            p->im2col_xoff.push_back(p->own_input ? (long long)(&m - p->models.data()) * input->B * input->in_h *
                                                        input->in_w * input->in_c * (long long)esz : 0);
            nd.im2col_idx = (int)p->im2col.size() - 1;
        }
    }
    for (Im2colProb& ip : p->im2col)
        fix.push_back({&ip.out, reserve((size_t)ip.B * ip.Ho * ip.Wo * ip.Kp * esz)});
    for (ModelInfo& m : p->models) {
        if (m.vacant) continue;
        {   // few classes: logits, loss and the input gradient of the last layer in one kernel
            const NodeInfo& last = m.nodes.back();
            const TensorInfo& hin = m.tensors[last.in_t];
            m.fused_head = !std::getenv("PACK_NO_FUSED_HEAD") && m.C <= HEAD_MAX_C && !hin.is_input &&
                           last.fan_in % (p->bf16 ? 8 : 4) == 0;
            if (m.fused_head) {
                const int nblk = (m.batch + HEAD_ROWS - 1) / HEAD_ROWS;
                fix.push_back({(void**)&m.head_partial, reserve((size_t)nblk * 4)});
            }
        }
        for (TensorInfo& t : m.tensors) {
            if (t.is_input) continue;
            fix.push_back({&t.act, reserve(t.elems() * (t.f32 ? 4 : esz))});
            fix.push_back({&t.dz, reserve((t.ld_dz ? (size_t)t.n * t.ld_dz : t.elems()) * esz)});
        }
        fix.push_back({(void**)&m.pred, reserve((size_t)m.batch * 4)});
    }
    const size_t loss_off = reserve((size_t)K * 4);
    const size_t err_off = reserve(4);
    const size_t zeros_off = reserve(256);
    TRY_ALLOC(p->slab, slab);
    p->slab_bytes = slab;
    for (auto& f : fix) *f.first = p->slab + f.second;
    p->loss_all = (float*)(p->slab + loss_off);
    p->err_flag = (int*)(p->slab + err_off);
    p->zeros = p->slab + zeros_off;
    for (int k = 0; k < K; ++k) p->models[k].loss = p->loss_all + k;

    DescBuilder db;
    size_t need = 0;
    build_plan(p, db, need);
    p->workspace_bytes = need;
    if (need) TRY_ALLOC(p->workspace, need);
    TRY_ALLOC(p->desc, db.bytes.size());
    p->desc_bytes = db.bytes.size();
#undef TRY_ALLOC
    if (p->dry) {
        p->desc_host.swap(db.bytes);
        return PACK_OK;
    }

    hipError_t e = hipMemcpy(p->desc, db.bytes.data(), db.bytes.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(p->slab, 0, p->slab_bytes);
    if (e == hipSuccess) e = hipMemset(p->grad, 0, p->arena_elems * 4);
    if (e == hipSuccess) e = hipMemset(p->master, 0, p->arena_elems * 4);
    if (e == hipSuccess && p->shadow) e = hipMemset(p->shadow, 0, p->arena_elems * 2);
    if (e == hipSuccess && p->opt_m) e = hipMemset(p->opt_m, 0, p->arena_elems * 4);
    if (e == hipSuccess && p->opt_v) e = hipMemset(p->opt_v, 0, p->arena_elems * 4);
    std::vector<long long> ends(K);
    for (int k = 0; k < K; ++k) ends[k] = (long long)p->models[k].arena_end;
    if (e == hipSuccess) e = hipMemcpy(p->seg_end, ends.data(), (size_t)K * sizeof(long long), hipMemcpyHostToDevice);
    if (e == hipSuccess && p->opt_params) {
        std::vector<OptStatic> par(K);
        for (int i = 0; i < K; ++i)
            par[i] = OptStatic{p->opt[i].kind, p->opt[i].mu, p->opt[i].beta1, p->opt[i].beta2, p->opt[i].eps};
        e = hipMemcpy(p->opt_params, par.data(), par.size() * sizeof(OptStatic), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        free_device(p);
        return fail(PACK_EDEVICE, std::string("initial upload: ") + hipGetErrorString(e));
    }
    return PACK_OK;
}

// seeded initial weights of member k: uniform in +-sqrt(6/fan_in), biases in +-1/sqrt(fan_in)
pack_status seed_weights(pack_ctx* p, int k, uint64_t seed) {
    ModelInfo& m = p->models[k];
    std::vector<float> blob(m.n_params);
    const bool bf16 = p->bf16;
    // every value is a hash of (seed, member, tensor, index): the ranges can be filled by several threads
    auto fill = [&](float* dst, size_t n, int tensor, float bound) {
        const size_t per = 1u << 18;
        const unsigned workers = (unsigned)std::min<size_t>(std::max(1u, std::min(16u, std::thread::hardware_concurrency())), (n + per - 1) / per);
        auto work = [=](size_t lo, size_t hi) {
            for (size_t i = lo; i < hi; ++i) {
                const float v = uniform_pm(seed, k, tensor, i, bound);
                dst[i] = bf16 ? round_to_bf16(v) : v;
            }
        };
        if (workers <= 1) { work(0, n); return; }
        std::vector<std::thread> pool;
        const size_t step = (n + workers - 1) / workers;
        size_t started = 0;   // elements handed to threads so far
        try {
            for (unsigned t = 0; t < workers; ++t) {
                pool.emplace_back(work, std::min(n, t * step), std::min(n, (t + 1) * step));
                started = std::min(n, (t + 1) * step);
            }
        } catch (const std::system_error&) {
            // no more threads to be had: this thread fills the rest
        }
        work(started, n);
        for (std::thread& t : pool) t.join();
    };
    int tensor = 0;
    for (const NodeInfo& nd : m.nodes) {
        if (nd.kind == NODE_GAP) continue;
        const float bw = std::sqrt(6.0f / (float)nd.fan_in), bb = 1.0f / std::sqrt((float)nd.fan_in);
        fill(blob.data() + nd.blob_off, nd.w_elems, tensor, bw);
        fill(blob.data() + nd.blob_off + nd.w_elems, (size_t)nd.out, tensor + 1, bb);
        tensor += 2;
    }
    return upload_weights(p, k, blob.data());
}

// What a slot of the pack shall hold after a change of membership or batch sizes.
struct SlotPlan {
    bool vacant = true;
    std::vector<pack_layer> layers;
    int batch = 0;
    int from = -1;   // slot of the current pack whose weights and optimiser state move in; -1: a new member
};

// Rebuilds the pack for `slots` and a shared batch of B rows.  A second pack is built beside the
// current one (so that a failure leaves the current one untouched), the state of every member that
// stays is copied over on the device, bit for bit, and the two change places.
pack_status rebuild(pack_ctx* p, int B, const std::vector<SlotPlan>& slots, uint64_t seed, int own_input = -1) {
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    pack_ctx* q = new (std::nothrow) pack_ctx();
    if (!q) return fail(PACK_ENOMEM, "host allocation failed");
    q->device = p->device;
    q->stream = p->stream;
    q->bf16 = p->bf16;
    q->in = p->in;
    q->in.B = B;
    q->own_input = own_input < 0 ? p->own_input : own_input != 0;
    q->keep_grads = p->keep_grads;
    q->K = (int)slots.size();
    q->models.resize(q->K);
    q->opt.assign(q->K, pack_opt_spec{PACK_OPT_SGD, 0.f, 0.f, 0.f, 0.f, 0.f});
    q->opt_t.assign(q->K, 0);
    for (int k = 0; k < q->K; ++k) {
        const SlotPlan& sp = slots[k];
        if (sp.vacant) {
            q->models[k].vacant = true;
            continue;
        }
        pack_model_spec spec{sp.layers.data(), (int32_t)sp.layers.size(), sp.batch};
        pack_status s = parse_model(q->in, spec, k, q->models[k]);
        if (s != PACK_OK) { release(q); return s; }
        if (sp.from >= 0) {
            q->opt[k] = p->opt[sp.from];
            q->opt_t[k] = p->opt_t[sp.from];
        }
    }
    pack_status s = build_device(q);
    if (s != PACK_OK) { release(q); return s; }
    hipError_t e = hipSuccess;
    for (int k = 0; k < q->K && e == hipSuccess; ++k) {
        const int f = slots[k].vacant ? -1 : slots[k].from;
        if (f < 0) continue;
        const ModelInfo& a = p->models[f];
        const ModelInfo& b = q->models[k];
        const size_t n = a.arena_end - a.arena_begin;
        if (n != b.arena_end - b.arena_begin) { release(q); return fail(PACK_EINVAL, "internal: member layout changed"); }
        e = hipMemcpyAsync(q->master + b.arena_begin, p->master + a.arena_begin, n * 4, hipMemcpyDeviceToDevice, p->stream);
        if (e == hipSuccess && p->shadow)
            e = hipMemcpyAsync((char*)q->shadow + b.arena_begin * 2, (const char*)p->shadow + a.arena_begin * 2, n * 2,
                               hipMemcpyDeviceToDevice, p->stream);
        if (e == hipSuccess && p->opt_m && q->opt_m)
            e = hipMemcpyAsync(q->opt_m + b.arena_begin, p->opt_m + a.arena_begin, n * 4, hipMemcpyDeviceToDevice, p->stream);
        if (e == hipSuccess && p->opt_v && q->opt_v)
            e = hipMemcpyAsync(q->opt_v + b.arena_begin, p->opt_v + a.arena_begin, n * 4, hipMemcpyDeviceToDevice, p->stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(p->stream);
    if (e != hipSuccess) { release(q); return fail(PACK_EDEVICE, std::string("moving member state: ") + hipGetErrorString(e)); }
    for (int k = 0; k < q->K; ++k) {
        if (slots[k].vacant || slots[k].from >= 0) continue;
        s = seed_weights(q, k, seed);
        if (s != PACK_OK) { release(q); return s; }
    }
    std::swap(*p, *q);
    release(q);   // the previous buffers
    return PACK_OK;
}

// the current pack as a list of slots that all stay where they are
std::vector<SlotPlan> current_slots(const pack_ctx* p) {
    std::vector<SlotPlan> slots(p->K);
    for (int k = 0; k < p->K; ++k) {
        const ModelInfo& m = p->models[k];
        slots[k].vacant = m.vacant;
        if (m.vacant) continue;
        slots[k].layers = m.layers;
        slots[k].batch = m.batch;
        slots[k].from = k;
    }
    return slots;
}

pack_status live_member(const pack_ctx* p, int32_t k) {
    if (!p) return fail(PACK_EINVAL, "null argument");
    if (k < 0 || k >= p->K) return fail(PACK_EINVAL, "member index out of range");
    if (p->models[k].vacant) return fail(PACK_EINVAL, "slot " + std::to_string(k) + " holds no member");
    return PACK_OK;
}

}  // namespace

extern "C" {

const char* pack_last_error(void) { return g_err.c_str(); }

pack_status pack_create(const pack_input_spec* input, const pack_model_spec* models, int32_t K,
                        uint64_t seed, void* hip_stream, pack_t** out) {
    if (out) *out = nullptr;
    if (!input || !models || !out) return fail(PACK_EINVAL, "null argument");
    if (K < 1 || K > PACK_MAX_MODELS) return fail(PACK_EINVAL, "K must be in [1, PACK_MAX_MODELS]");
    if (input->B < 1 || input->in_h < 1 || input->in_w < 1 || input->in_c < 1) return fail(PACK_EINVAL, "bad input shape");
    if (input->dtype != PACK_F32 && input->dtype != PACK_BF16) return fail(PACK_EINVAL, "unknown dtype");

    pack_ctx* p = new (std::nothrow) pack_ctx();
    if (!p) return fail(PACK_ENOMEM, "host allocation failed");
    p->stream = (hipStream_t)hip_stream;
    p->bf16 = (input->dtype == PACK_BF16);
    p->K = K;
    p->in = *input;
    p->models.resize(K);
    p->opt.assign(K, pack_opt_spec{PACK_OPT_SGD, 0.f, 0.f, 0.f, 0.f, 0.f});
    p->opt_t.assign(K, 0);
    for (int k = 0; k < K; ++k) {
        pack_status s = parse_model(*input, models[k], k, p->models[k]);
        if (s != PACK_OK) { release(p); return s; }
    }
    if (hipGetDevice(&p->device) != hipSuccess) {
        (void)hipGetLastError();
        release(p);
        return fail(PACK_EDEVICE, "no HIP device is current");
    }
    pack_status s = build_device(p);
    if (s != PACK_OK) { release(p); return s; }
    for (int k = 0; k < K; ++k) {
        s = seed_weights(p, k, seed);
        if (s != PACK_OK) { release(p); return s; }
    }
    *out = p;
    return PACK_OK;
}

pack_status pack_plan_check(const pack_input_spec* input, const pack_model_spec* models, int32_t K, int32_t input_mode,
                            int64_t* launches_walked, int64_t* launches_skipped, int64_t* loads_checked) {
    if (!input || !models) return fail(PACK_EINVAL, "null argument");
    if (K < 1 || K > PACK_MAX_MODELS) return fail(PACK_EINVAL, "K must be in [1, PACK_MAX_MODELS]");
    if (input->B < 1 || input->in_h < 1 || input->in_w < 1 || input->in_c < 1) return fail(PACK_EINVAL, "bad input shape");
    if (input->dtype != PACK_F32 && input->dtype != PACK_BF16) return fail(PACK_EINVAL, "unknown dtype");
    if (input_mode != PACK_INPUT_SHARED && input_mode != PACK_INPUT_PER_MEMBER) return fail(PACK_EINVAL, "unknown input mode");
    pack_ctx* p = new (std::nothrow) pack_ctx();
    if (!p) return fail(PACK_ENOMEM, "host allocation failed");
    p->dry = true;
    p->bf16 = (input->dtype == PACK_BF16);
    p->K = K;
    p->in = *input;
    p->own_input = input_mode == PACK_INPUT_PER_MEMBER;
    p->models.resize(K);
    p->opt.assign(K, pack_opt_spec{PACK_OPT_SGD, 0.f, 0.f, 0.f, 0.f, 0.f});
    p->opt_t.assign(K, 0);
    for (int k = 0; k < K; ++k) {
        pack_status s = parse_model(*input, models[k], k, p->models[k]);
        if (s != PACK_OK) { release(p); return s; }
    }
    pack_status s = build_device(p);
    if (s != PACK_OK) { release(p); return s; }
    // the step's input: one more made-up allocation
    const size_t esz = p->bf16 ? 2 : 4;
    const size_t x_bytes = (size_t)input->B * input->in_h * input->in_w * input->in_c * esz * (p->own_input ? (size_t)K : 1);
    void* x_fake = nullptr;
    (void)dev_alloc(&x_fake, x_bytes, p);
    auto region_holds = [&](const void* ptr, long long bytes) {
        const uintptr_t a = (uintptr_t)ptr;
        for (const auto& r : p->dry_regions)
            if (a >= r.first && a + (uintptr_t)bytes <= r.first + r.second) return true;
        return false;
    };
    long long walked = 0, skipped = 0, loads = 0, frags = 0;
    std::string err;
    for (size_t li = 0; li < p->plan.size() && err.empty(); ++li) {
        const Launch& L = p->plan[li];
        if (L.kind != L_GEMM) continue;
        const bool halo = L.mode == CONV_DW && is_halo_cfg(L.tile_cfg);
        const bool rows = (L.mode == CONV_FWD || L.mode == CONV_DX) && is_rows_cfg(L.tile_cfg);
        const int ci_t = halo ? GEMM_TILE_N[L.tile_cfg] / 9 : 0;      // input channels per tile
        const bool staged = !halo && !rows && L.tile_cfg != GEMM_CFG_SCALAR;
        if (!halo && !rows && !staged) { ++skipped; continue; }      // the element-by-element kernels load by the definition itself
        ++walked;
        const GemmProb* probs = (const GemmProb*)(p->desc_host.data() + L.desc_off);
        const TileRef* tiles = (const TileRef*)(p->desc_host.data() + L.map_off);
        if (staged) {
            // aligned staged-tile kernels: the fetchers themselves, run on the CPU, against the definition of the operands
            const int BMc = GEMM_TILE_M[L.tile_cfg], BNc = GEMM_TILE_N[L.tile_cfg];
            std::map<std::vector<int>, int> dealt;
            int n_probs = 0;
            for (int t = 0; t < L.n && err.empty(); ++t) {
                const TileRef& tr = tiles[t];
                if (tr.prob < 0) continue;
                n_probs = std::max(n_probs, tr.prob + 1);
                GemmProb g = probs[tr.prob];
                if (g.flags & F_A_INPUT) g.A = (const char*)x_fake + g.x_off;
                if (g.flags & F_B_INPUT) g.B = (const char*)x_fake + g.x_off;
                unsigned long long alo, ahi, blo, bhi;
                err = gemm_fetch_walk(p->bf16, L.mode, BMc, BNc, g, tr, &alo, &ahi, &blo, &bhi, &loads);
                if (err.empty() && alo < ahi && !region_holds((const void*)(uintptr_t)alo, (long long)(ahi - alo))) err = "the loads of operand A are not inside one allocation";
                if (err.empty() && blo < bhi && !region_holds((const void*)(uintptr_t)blo, (long long)(bhi - blo))) err = "the loads of operand B are not inside one allocation";
                if (++dealt[{tr.prob, tr.tm, tr.tn, tr.ks}] > 1 && err.empty()) err = "a tile is dealt twice";
                if (!err.empty()) err = "launch " + std::to_string(li) + " (mode " + std::to_string(L.mode) + "), tile " + std::to_string(t) + " (problem " + std::to_string(tr.prob) +
                                        ", tm " + std::to_string(tr.tm) + ", tn " + std::to_string(tr.tn) + ", split " + std::to_string(tr.ks) + "): " + err;
            }
            for (int i = 0; i < n_probs && err.empty(); ++i) {
                const GemmProb& g = probs[i];
                const int S = std::max(1, (g.Kd + g.ksplit - 1) / g.ksplit);
                for (int ks = 0; ks < S; ++ks)
                    for (int tm = 0; tm < (g.R + BMc - 1) / BMc; ++tm)
                        for (int tn = 0; tn < (g.Q + BNc - 1) / BNc; ++tn)
                            if (dealt.find({i, tm, tn, ks}) == dealt.end() && err.empty())
                                err = "launch " + std::to_string(li) + ": problem " + std::to_string(i) + " lacks a tile";
            }
            continue;
        }
        if (rows) {
            // stride-1 forward / input gradient, halo form: the gathered operand of every tile, and every tile once
            const int BMc = GEMM_TILE_M[L.tile_cfg], BNc = GEMM_TILE_N[L.tile_cfg];
            const bool dx = L.mode == CONV_DX;
            std::map<std::vector<int>, int> dealt;
            int n_probs = 0;
            for (int t = 0; t < L.n && err.empty(); ++t) {
                const TileRef& tr = tiles[t];
                if (tr.prob < 0) continue;
                n_probs = std::max(n_probs, tr.prob + 1);
                const GemmProb& g = probs[tr.prob];
                const long long a_bytes = (long long)g.R * (dx ? g.Cout : g.Cin) * (long long)esz;
                if (!region_holds(g.A, a_bytes)) err = "the gathered operand is not inside one allocation";
                if (err.empty() && (tr.ks != 0 || tr.tm < 0 || tr.tm >= g.R / BMc || tr.tn < 0 || tr.tn >= (g.Q + BNc - 1) / BNc)) err = "a tile lies outside its problem";
                // (the gathered operand does not depend on the column tile: walked once per row tile)
                if (err.empty() && tr.tn == 0) err = conv_rows_halo_walk(p->bf16, L.tile_cfg == GEMM_CFG_ROWS32, dx, g, tr, a_bytes, &loads, &frags);
                if (++dealt[{tr.prob, tr.tm, tr.tn}] > 1 && err.empty()) err = "a tile is dealt twice";
                if (!err.empty()) err = "launch " + std::to_string(li) + ", tile " + std::to_string(t) + " (problem " + std::to_string(tr.prob) + ", tm " +
                                        std::to_string(tr.tm) + ", tn " + std::to_string(tr.tn) + "): " + err;
            }
            for (int i = 0; i < n_probs && err.empty(); ++i)
                for (int tm = 0; tm < probs[i].R / BMc; ++tm)
                    for (int tn = 0; tn < (probs[i].Q + BNc - 1) / BNc; ++tn)
                        if (dealt.find({i, tm, tn}) == dealt.end() && err.empty())
                            err = "launch " + std::to_string(li) + ": problem " + std::to_string(i) + " lacks a tile";
            continue;
        }
        std::map<std::vector<int>, int> seen;          // (problem, tm, tn, ks) -> times dealt
        int n_probs = 0;
        for (int t = 0; t < L.n && err.empty(); ++t) {
            const TileRef& tr = tiles[t];
            if (tr.prob < 0) continue;
            n_probs = std::max(n_probs, tr.prob + 1);
            GemmProb g = probs[tr.prob];
            if (g.flags & F_B_INPUT) g.B = (const char*)x_fake + g.x_off;
            const long long a_bytes = (long long)g.Kd * g.Cout * (long long)esz;
            const long long b_bytes = (long long)(g.Kd / (g.Ho * g.Wo)) * g.H * g.W * g.Cin * (long long)esz;
            if (!region_holds(g.A, a_bytes) || !region_holds(g.B, b_bytes)) err = "an operand of a weight-gradient problem is not inside one allocation";
            const long long out_bytes = (long long)g.Cout * g.ldc * 4;
            const char* out_base = (g.flags & F_WS) ? p->workspace + (size_t)(uintptr_t)g.C : (const char*)g.C;
            if (err.empty() && !region_holds(out_base + (long long)tr.ks * g.split_stride * 4, out_bytes)) err = "a weight-gradient output is not inside one allocation";
            if (err.empty()) err = conv_dw_halo_walk(p->bf16, ci_t == 64, g, tr, a_bytes, b_bytes, false, &loads, &frags);
            if (++seen[{tr.prob, tr.tm, tr.tn, tr.ks}] > 1 && err.empty()) err = "a tile is dealt twice";
            if (!err.empty()) err = "launch " + std::to_string(li) + ", tile " + std::to_string(t) + " (problem " + std::to_string(tr.prob) + ", tm " +
                                    std::to_string(tr.tm) + ", tn " + std::to_string(tr.tn) + ", split " + std::to_string(tr.ks) + "): " + err;
        }
        for (int i = 0; i < n_probs && err.empty(); ++i) {
            const GemmProb& g = probs[i];
            const int S = (g.Kd + g.ksplit - 1) / g.ksplit;
            for (int ks = 0; ks < S; ++ks)
                for (int tm = 0; tm < g.Cout / 64; ++tm)
                    for (int tn = 0; tn < g.Cin / ci_t; ++tn)
                        if (seen.find({i, tm, tn, ks}) == seen.end() && err.empty())
                            err = "launch " + std::to_string(li) + ": problem " + std::to_string(i) + " lacks a tile";
        }
    }
    release(p);
    if (launches_walked) *launches_walked = walked;
    if (launches_skipped) *launches_skipped = skipped;
    if (loads_checked) *loads_checked = loads + frags;
    if (!err.empty()) return fail(PACK_EINVAL, "plan check: " + err);
    return PACK_OK;
}

pack_status pack_free(pack_t* p, int32_t k) {
    pack_status s = live_member(p, k);
    if (s != PACK_OK) return s;
    std::vector<SlotPlan> slots = current_slots(p);
    slots[k] = SlotPlan{};
    return rebuild(p, p->in.B, slots, 0);
}

pack_status pack_load(pack_t* p, const pack_model_spec* model, uint64_t seed, int32_t* k_out) {
    if (!p || !model || !k_out) return fail(PACK_EINVAL, "null argument");
    if (!model->layers || model->n_layers < 1) return fail(PACK_EINVAL, "empty layer list");
    std::vector<SlotPlan> slots = current_slots(p);
    int k = 0;
    while (k < (int)slots.size() && !slots[k].vacant) ++k;
    if (k == (int)slots.size()) {
        if (k >= PACK_MAX_MODELS) return fail(PACK_EINVAL, "the pack already has PACK_MAX_MODELS members");
        slots.push_back(SlotPlan{});
    }
    slots[k].vacant = false;
    slots[k].layers.assign(model->layers, model->layers + model->n_layers);
    slots[k].batch = model->batch;
    slots[k].from = -1;
    pack_status s = rebuild(p, p->in.B, slots, seed);
    if (s == PACK_OK) *k_out = k;
    return s;
}

pack_status pack_set_batch(pack_t* p, int32_t B, const int32_t* batch) {
    if (!p || !batch) return fail(PACK_EINVAL, "null argument");
    if (B < 1) return fail(PACK_EINVAL, "B < 1");
    std::vector<SlotPlan> slots = current_slots(p);
    bool same = (B == p->in.B);
    for (int k = 0; k < p->K; ++k) {
        if (slots[k].vacant) continue;
        if (batch[k] < 1 || batch[k] > B) return fail(PACK_EINVAL, "member " + std::to_string(k) + ": batch outside [1, B]");
        if (batch[k] != slots[k].batch) same = false;
        slots[k].batch = batch[k];
    }
    if (same) return PACK_OK;
    return rebuild(p, B, slots, 0);
}

pack_status pack_set_input_mode(pack_t* p, int32_t mode) {
    if (!p) return fail(PACK_EINVAL, "null argument");
    if (mode != PACK_INPUT_SHARED && mode != PACK_INPUT_PER_MEMBER) return fail(PACK_EINVAL, "unknown input mode");
    if ((mode == PACK_INPUT_PER_MEMBER) == p->own_input) return PACK_OK;
    return rebuild(p, p->in.B, current_slots(p), 0, mode == PACK_INPUT_PER_MEMBER ? 1 : 0);
}

size_t pack_estimate_bytes(const pack_input_spec* input, const pack_model_spec* model, int32_t opt_kind) {
    if (!input || !model || input->B < 1 || input->in_h < 1 || input->in_w < 1 || input->in_c < 1) return 0;
    if (input->dtype != PACK_F32 && input->dtype != PACK_BF16) return 0;
    if (opt_kind < PACK_OPT_SGD || opt_kind > PACK_OPT_ADAM) return 0;
    ModelInfo m;
    if (parse_model(*input, *model, 0, m) != PACK_OK) return 0;
    const bool bf = input->dtype == PACK_BF16;
    const size_t esz = bf ? 2 : 4;
    size_t arena = 0, wt = 0, slab = 0;
    for (const NodeInfo& nd : m.nodes) {
        if (nd.kind == NODE_GAP) continue;
        arena = align_up(arena + nd.w_arena, 64);
        arena = align_up(arena + (size_t)nd.out, 64);
        if (nd.kind == NODE_CONV && !nd.kp && m.tensors[nd.in_t].needs_grad) wt = align_up(wt + nd.w_elems, 64);
    }
    for (const TensorInfo& t : m.tensors) {
        if (t.is_input) continue;
        slab += align_up(t.elems() * (t.f32 ? 4 : esz), 256);
        slab += align_up((t.ld_dz ? (size_t)t.n * t.ld_dz : t.elems()) * esz, 256);
    }
    slab += align_up((size_t)m.batch * 4, 256);
    const size_t states = opt_kind == PACK_OPT_SGD ? 0 : opt_kind == PACK_OPT_ADAM ? 2 : 1;
    return arena * (4 + 4 + (bf ? 2 : 0) + 4 * states) + wt * esz + slab;
}

int32_t pack_num_slots(const pack_t* p) { return p ? p->K : 0; }

int32_t pack_member_batch(const pack_t* p, int32_t k) {
    if (!p || k < 0 || k >= p->K || p->models[k].vacant) return 0;
    return p->models[k].batch;
}

pack_status pack_write_weights(pack_t* p, int32_t k, const float* host_src, size_t n_floats) {
    if (!p || !host_src) return fail(PACK_EINVAL, "null argument");
    pack_status st = live_member(p, k);
    if (st != PACK_OK) return st;
    if (n_floats != p->models[k].n_params) return fail(PACK_EINVAL, "n_floats does not match pack_num_params");
    return upload_weights(p, k, host_src);
}

// one training step with the partial sums of split weight gradients in `ws`
static pack_status step_with_workspace(pack_t* p, const void* x_dev, const int32_t* labels_dev, const float* lr_host, char* ws) {
    if (((uintptr_t)x_dev & 15) || ((uintptr_t)labels_dev & 3)) return fail(PACK_EINVAL, "x_dev must be 16-byte aligned");
    LrTable lr;
    for (int k = 0; k < PACK_LR_N; ++k) lr.lr[k] = (k < p->K) ? lr_host[k] : 0.f;
    const bool bf = p->bf16;
    const bool timed_step = p->profiling && (p->profile_step++ % p->profile_every == 0);
    for (size_t li = 0; li < p->plan.size(); ++li) {
        const Launch& L = p->plan[li];
        hipError_t e = hipSuccess;
        const bool timed = timed_step && (p->profile_which < 0 || p->profile_which == (int)li);
        pack_ctx::Stamp stamp{(int)li, nullptr, nullptr};
        if (timed) {
            if (hipEventCreate(&stamp.t0) != hipSuccess || hipEventCreate(&stamp.t1) != hipSuccess ||
                hipEventRecord(stamp.t0, p->stream) != hipSuccess)
                return fail(PACK_EDEVICE, "profiling event");
        }
        const char* d = p->desc + L.desc_off;
        const char* mp = p->desc + L.map_off;
        switch (L.kind) {
            case L_GEMM:
                e = launch_gemm(L.mode, bf, L.tile_cfg, (const GemmProb*)d, (const TileRef*)mp, L.n, x_dev, ws, lr, p->stream);
                break;
            case L_REDUCE: e = launch_reduce((const ReduceProb*)d, (const int2*)mp, L.n, ws, lr, p->stream); break;
            case L_CE: e = launch_ce(bf, (const CeProb*)d, L.n, labels_dev, p->err_flag, p->stream); break;
            case L_HEAD: e = launch_head(bf, L.mode, (const HeadProb*)d, (const int2*)mp, L.n, labels_dev, p->err_flag, p->stream); break;
            case L_GAP_FWD: e = launch_gap(bf, false, (const GapProb*)d, (const int2*)mp, L.n, p->stream); break;
            case L_GAP_BWD: e = launch_gap(bf, true, (const GapProb*)d, (const int2*)mp, L.n, p->stream); break;
            case L_SHORTCUT: e = launch_shortcut_bwd(bf, (const ShortcutProb*)d, (const int2*)mp, L.n, p->stream); break;
            case L_IM2COL: e = launch_im2col(bf, p->im2col[L.mode], (const char*)x_dev + p->im2col_xoff[L.mode], p->stream); break;
            case L_WTRANS: e = launch_wtranspose(bf, (const TransposeProb*)d, (const int2*)mp, L.n, p->stream); break;
            case L_SGD:
                if (!p->any_opt) {
                    e = launch_sgd(p->master, p->grad, p->shadow, (long long)p->arena_elems, p->seg_end, p->K, lr, p->stream);
                } else {
                    OptTable tab;
                    for (int k = 0; k < 256; ++k) {
                        tab.lr[k] = (k < p->K) ? lr_host[k] : 0.f;
                        tab.c1[k] = tab.c2[k] = 1.f;
                        if (k < p->K && p->opt[k].kind == PACK_OPT_ADAM) {
                            const double t = (double)(p->opt_t[k] + 1);
                            tab.c1[k] = (float)(1.0 / (1.0 - std::pow((double)p->opt[k].beta1, t)));
                            tab.c2[k] = (float)(1.0 / (1.0 - std::pow((double)p->opt[k].beta2, t)));
                        }
                    }
                    e = launch_opt(p->master, p->grad, p->shadow, p->opt_m, p->opt_v, (long long)p->arena_elems,
                                   p->seg_end, p->opt_params, p->K, tab, p->stream);
                    if (e == hipSuccess)
                        for (int k = 0; k < p->K; ++k) ++p->opt_t[k];
                }
                break;
        }
        if (e != hipSuccess) return fail(PACK_EDEVICE, std::string("kernel launch: ") + hipGetErrorString(e));
        if (timed) {
            if (hipEventRecord(stamp.t1, p->stream) != hipSuccess) return fail(PACK_EDEVICE, "profiling event");
            p->stamps.push_back(stamp);
        }
    }
    return PACK_OK;
}

pack_status pack_step(pack_t* p, const void* x_dev, const int32_t* labels_dev, const float* lr_host) {
    if (!p || !x_dev || !labels_dev || !lr_host) return fail(PACK_EINVAL, "null argument");
    return step_with_workspace(p, x_dev, labels_dev, lr_host, p->workspace);
}

size_t pack_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

size_t pack_workspace_bytes(const pack_t* p) { return p ? p->workspace_bytes : 0; }

pack_status pack_step_static(pack_t* p, const void* x_dev, const int32_t* labels_dev, const float* lr_host) {
    if (!p || !x_dev || !labels_dev || !lr_host) return fail(PACK_EINVAL, "null argument");
    if (p->profiling) return fail(PACK_EINVAL, "pack_step_static does not time launches (events are allocations): call pack_profile_stop first");
    if (p->workspace_bytes > STATIC_SCRATCH_BYTES)
        return fail(PACK_ENOMEM, "the pack's split weight gradients need " + std::to_string(p->workspace_bytes) +
                                 " bytes of scratch, the library's static array holds " + std::to_string(STATIC_SCRATCH_BYTES));
    // the array's address on this device, looked up once per device (every GPU holds its own copy)
    static std::mutex mu;
    static char* scratch_of[64] = {nullptr};
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev), PACK_EDEVICE);
    if (dev < 0 || dev >= 64) return fail(PACK_EDEVICE, "device index outside [0, 64)");
    if (dev != p->device) return fail(PACK_EINVAL, "the pack was created on another device than the current one");
    char* ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!scratch_of[dev]) HIP_TRY(static_scratch(&scratch_of[dev]), PACK_EDEVICE);
        ws = scratch_of[dev];
    }
    if (!ws) return fail(PACK_EDEVICE, "no address for the static scratch array");
    return step_with_workspace(p, x_dev, labels_dev, lr_host, ws);
}

pack_status pack_profile_start(pack_t* p, int32_t which, int32_t every) {
    if (!p || every < 1) return fail(PACK_EINVAL, "null argument or every < 1");
    if (which >= (int32_t)p->plan.size()) return fail(PACK_EINVAL, "launch index out of range");
    for (auto& s : p->stamps) { (void)hipEventDestroy(s.t0); (void)hipEventDestroy(s.t1); }
    p->stamps.clear();
    p->profiling = true;
    p->profile_which = which;
    p->profile_every = every;
    p->profile_step = 0;
    return PACK_OK;
}

pack_status pack_profile_stop(pack_t* p, float* ms_sum, int32_t* count) {
    if (!p || !ms_sum || !count) return fail(PACK_EINVAL, "null argument");
    p->profiling = false;
    for (size_t i = 0; i < p->plan.size(); ++i) { ms_sum[i] = 0.f; count[i] = 0; }
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    pack_status st = PACK_OK;
    for (auto& s : p->stamps) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, s.t0, s.t1) == hipSuccess) { ms_sum[s.launch] += ms; count[s.launch] += 1; }
        else st = fail(PACK_EDEVICE, "hipEventElapsedTime failed");
        (void)hipEventDestroy(s.t0);
        (void)hipEventDestroy(s.t1);
    }
    p->stamps.clear();
    return st;
}

pack_status pack_launch_name(const pack_t* p, int32_t i, char* buf, size_t n) {
    if (!p || !buf || n == 0) return fail(PACK_EINVAL, "null argument");
    if (i < 0 || i >= (int32_t)p->plan.size()) return fail(PACK_EINVAL, "launch index out of range");
    static const char* gemm_names[] = {"gemm_lin_fwd", "gemm_lin_dx", "gemm_lin_dw", "gemm_conv_fwd", "gemm_conv_dx", "gemm_conv_dw"};
    static const char* names[] = {"", "reduce_partials", "softmax_xent", "gap_fwd", "gap_bwd", "shortcut_bwd", "sgd_update", "im2col_shared_input", "transpose_conv_weights", "classifier_head"};
    const Launch& L = p->plan[i];
    const char* nm = (L.kind == L_GEMM) ? gemm_names[L.mode] : names[L.kind];
    if (L.kind == L_SGD && p->any_opt) nm = "optimizer_update";
    const bool with_update = p->fused && (L.kind == L_REDUCE || (L.kind == L_GEMM && (L.mode == LIN_DW || L.mode == CONV_DW)));
    std::snprintf(buf, n, "%s%s", nm, with_update ? "+sgd" : "");
    return PACK_OK;
}

pack_status pack_launch_flops(const pack_t* p, int32_t i, double* flops) {
    if (!p || !flops) return fail(PACK_EINVAL, "null argument");
    if (i < 0 || i >= (int32_t)p->plan.size()) return fail(PACK_EINVAL, "launch index out of range");
    *flops = p->plan[i].flops;
    return PACK_OK;
}

pack_status pack_launch_bytes(const pack_t* p, int32_t i, double* bytes) {
    if (!p || !bytes) return fail(PACK_EINVAL, "null argument");
    if (i < 0 || i >= (int32_t)p->plan.size()) return fail(PACK_EINVAL, "launch index out of range");
    *bytes = p->plan[i].bytes;
    return PACK_OK;
}

pack_status pack_launch_tile(const pack_t* p, int32_t i, int32_t* tile_rows, int32_t* tile_cols, int32_t* lean) {
    if (!p || !tile_rows || !tile_cols || !lean) return fail(PACK_EINVAL, "null argument");
    if (i < 0 || i >= (int32_t)p->plan.size()) return fail(PACK_EINVAL, "launch index out of range");
    const Launch& L = p->plan[i];
    const bool gemm = L.kind == L_GEMM;
    *tile_rows = gemm ? GEMM_TILE_M[L.tile_cfg] : 0;
    *tile_cols = gemm ? GEMM_TILE_N[L.tile_cfg] : 0;
    *lean = gemm && (L.tile_cfg == GEMM_CFG_LEAN || L.tile_cfg == GEMM_CFG_LEAN64);
    return PACK_OK;
}

pack_status pack_keep_grads(pack_t* p, int32_t on) {
    if (!p) return fail(PACK_EINVAL, "null argument");
    if ((on != 0) == p->keep_grads) return PACK_OK;
    p->keep_grads = (on != 0);
    pack_status st = rebuild(p, p->in.B, current_slots(p), 0);
    if (st != PACK_OK) p->keep_grads = !p->keep_grads;
    return st;
}

pack_status pack_set_optimizer(pack_t* p, int32_t k, const pack_opt_spec* spec) {
    if (!p || !spec) return fail(PACK_EINVAL, "null argument");
    {
        pack_status lm = live_member(p, k);
        if (lm != PACK_OK) return lm;
    }
    const pack_opt_spec o = *spec;
    auto unit = [](float v) { return v >= 0.f && v < 1.f; };
    switch (o.kind) {
        case PACK_OPT_SGD: break;
        case PACK_OPT_MOMENTUM: if (!unit(o.mu)) return fail(PACK_EINVAL, "momentum must be in [0, 1)"); break;
        case PACK_OPT_ADAGRAD: if (!(o.acc0 > 0.f)) return fail(PACK_EINVAL, "initial accumulator must be > 0"); break;
        case PACK_OPT_ADAM:
            if (!unit(o.beta1) || !unit(o.beta2) || !(o.eps > 0.f)) return fail(PACK_EINVAL, "beta1, beta2 in [0, 1) and eps > 0");
            break;
        default: return fail(PACK_EINVAL, "unknown optimiser kind");
    }
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    const pack_opt_spec old_spec = p->opt[k];
    const long long old_t = p->opt_t[k];
    p->opt[k] = o;
    p->opt_t[k] = 0;
    bool need_m = false, need_v = false;
    for (const pack_opt_spec& q : p->opt) {
        if (q.kind != PACK_OPT_SGD) need_m = true;
        if (q.kind == PACK_OPT_ADAM) need_v = true;
    }
    if (need_m != (p->opt_m != nullptr) || need_v != (p->opt_v != nullptr) || need_m != p->any_opt) {
        // the set of state arrays, or whether the update is fused into the weight-gradient kernels,
        // changes: plan the pack again (members keep their weights and state)
        pack_status st = rebuild(p, p->in.B, current_slots(p), 0);
        if (st != PACK_OK) {
            p->opt[k] = old_spec;
            p->opt_t[k] = old_t;
            return st;
        }
    } else if (p->opt_params) {
        std::vector<OptStatic> par(p->K);
        for (int i = 0; i < p->K; ++i)
            par[i] = OptStatic{p->opt[i].kind, p->opt[i].mu, p->opt[i].beta1, p->opt[i].beta2, p->opt[i].eps};
        HIP_TRY(hipMemcpy(p->opt_params, par.data(), par.size() * sizeof(OptStatic), hipMemcpyHostToDevice), PACK_EDEVICE);
    }
    // starting state over the member's whole arena segment (alignment gaps included: their gradient
    // is always zero, and a positive Adagrad accumulator there keeps 0 / sqrt(acc) well defined)
    const ModelInfo& m = p->models[k];
    const size_t seg = m.arena_end - m.arena_begin;
    if (p->opt_m) {
        std::vector<float> init(seg, o.kind == PACK_OPT_ADAGRAD ? o.acc0 : 0.f);
        HIP_TRY(hipMemcpy(p->opt_m + m.arena_begin, init.data(), seg * 4, hipMemcpyHostToDevice), PACK_EDEVICE);
    }
    if (p->opt_v) HIP_TRY(hipMemset(p->opt_v + m.arena_begin, 0, seg * 4), PACK_EDEVICE);
    return PACK_OK;
}

static pack_status opt_slot(pack_t* p, int32_t k, int32_t slot, float** arena) {
    pack_status lm = live_member(p, k);
    if (lm != PACK_OK) return lm;
    const int kind = p->opt[k].kind;
    const bool has = (slot == 0 && kind != PACK_OPT_SGD) || (slot == 1 && kind == PACK_OPT_ADAM);
    if (!has) return fail(PACK_EINVAL, "the member's optimiser has no such state array");
    *arena = slot == 0 ? p->opt_m : p->opt_v;
    return PACK_OK;
}

pack_status pack_read_opt_state(pack_t* p, int32_t k, int32_t slot, float* host_dst, size_t n_floats, int64_t* steps) {
    float* arena = nullptr;
    pack_status st = opt_slot(p, k, slot, &arena);
    if (st != PACK_OK) return st;
    st = download(p, k, arena, host_dst, n_floats);
    if (st == PACK_OK && steps) *steps = p->opt_t[k];
    return st;
}

pack_status pack_write_opt_state(pack_t* p, int32_t k, int32_t slot, const float* host_src, size_t n_floats, int64_t steps) {
    float* arena = nullptr;
    pack_status st = opt_slot(p, k, slot, &arena);
    if (st != PACK_OK) return st;
    if (!host_src || steps < 0) return fail(PACK_EINVAL, "null argument or negative step count");
    ModelInfo& m = p->models[k];
    if (n_floats != m.n_params) return fail(PACK_EINVAL, "n_floats does not match pack_num_params");
    std::vector<float> seg;
    blob_to_arena(m, host_src, seg);
    if (p->opt[k].kind == PACK_OPT_ADAGRAD && slot == 0) {
        // positions outside the blob (alignment gaps, padded columns) keep a positive accumulator
        std::vector<float> ones(m.n_params, 1.f), mark;
        blob_to_arena(m, ones.data(), mark);
        for (size_t i = 0; i < seg.size(); ++i)
            if (mark[i] == 0.f) seg[i] = p->opt[k].acc0;
    }
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    HIP_TRY(hipMemcpy(arena + m.arena_begin, seg.data(), seg.size() * 4, hipMemcpyHostToDevice), PACK_EDEVICE);
    p->opt_t[k] = steps;
    return PACK_OK;
}

pack_status pack_gather_batch(pack_t* p, const void* data_dev, const int32_t* labels_all_dev, int64_t n_samples,
                              const int64_t* idx_dev, int32_t rows, void* x_out_dev, int32_t* labels_out_dev) {
    if (!p || !data_dev || !labels_all_dev || !idx_dev || !x_out_dev || !labels_out_dev) return fail(PACK_EINVAL, "null argument");
    if (n_samples < 1) return fail(PACK_EINVAL, "n_samples < 1");
    if (rows < 0 || rows > p->in.B) return fail(PACK_EINVAL, "rows outside [0, B]");
    if (((uintptr_t)labels_all_dev & 3) || ((uintptr_t)labels_out_dev & 3) || ((uintptr_t)idx_dev & 7))
        return fail(PACK_EINVAL, "labels must be 4-byte aligned and indices 8-byte aligned");
    const long long row_bytes = (long long)p->in.in_h * p->in.in_w * p->in.in_c * (p->bf16 ? 2 : 4);
    if (((uintptr_t)data_dev | (uintptr_t)x_out_dev) & (p->bf16 ? 1 : 3)) return fail(PACK_EINVAL, "data pointers must be aligned to the element type");
    HIP_TRY(launch_gather_rows(data_dev, labels_all_dev, (const long long*)idx_dev, (long long)n_samples, rows, row_bytes,
                               x_out_dev, labels_out_dev, p->err_flag, p->stream), PACK_EDEVICE);
    return PACK_OK;
}

pack_status pack_measure_ceiling(int32_t what, void* stream, double* value_out) {
    if (!value_out) return fail(PACK_EINVAL, "null argument");
    if (what < PACK_CEILING_HBM_COPY || what > PACK_CEILING_MFMA_FP32) return fail(PACK_EINVAL, "unknown ceiling");
    hipStream_t st = (hipStream_t)stream;
    const long long copy_bytes = 1ll << 30;                  // far beyond every cache on the chip
    const int blocks = 256 * 8, iters = 20000, reps = 5;
    char* buf = nullptr;
    hipEvent_t t0 = nullptr, t1 = nullptr;
    const size_t need = what == PACK_CEILING_HBM_COPY ? (size_t)copy_bytes * 2 : (size_t)blocks * 256 * 4;
    auto cleanup = [&]() {
        if (t0) (void)hipEventDestroy(t0);
        if (t1) (void)hipEventDestroy(t1);
        if (buf) (void)hipFree(buf);
    };
    hipError_t e = hipMalloc((void**)&buf, need);
    if (e == hipSuccess) e = hipEventCreate(&t0);
    if (e == hipSuccess) e = hipEventCreate(&t1);
    double work = 0.0;                                       // bytes or flops of one launch
    auto once = [&]() -> hipError_t {
        if (what == PACK_CEILING_HBM_COPY) { work = 2.0 * (double)copy_bytes; return launch_ceiling_copy(buf, buf + copy_bytes, copy_bytes, st); }
        return launch_ceiling_mfma(what == PACK_CEILING_MFMA_BF16, (float*)buf, blocks, iters, &work, st);
    };
    if (e == hipSuccess && what == PACK_CEILING_HBM_COPY) e = launch_fill_zero(buf, copy_bytes, st);
    for (int i = 0; i < 2 && e == hipSuccess; ++i) e = once();          // warm-up
    if (e == hipSuccess) e = hipEventRecord(t0, st);
    for (int i = 0; i < reps && e == hipSuccess; ++i) e = once();
    if (e == hipSuccess) e = hipEventRecord(t1, st);
    if (e == hipSuccess) e = hipEventSynchronize(t1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
    cleanup();
    if (e != hipSuccess) return fail(PACK_EDEVICE, std::string("pack_measure_ceiling: ") + hipGetErrorString(e));
    if (!(ms > 0.0f)) return fail(PACK_EDEVICE, "pack_measure_ceiling: no time elapsed");
    const double per_s = work * reps / ((double)ms * 1e-3);
    *value_out = what == PACK_CEILING_HBM_COPY ? per_s / 1e9 : per_s / 1e12;
    return PACK_OK;
}

pack_status pack_read_loss(pack_t* p, float* host_dst) {
    if (!p || !host_dst) return fail(PACK_EINVAL, "null argument");
    // members with a fused classifier head leave per-block sums; add them up now, in block order
    if (p->n_heads) HIP_TRY(launch_head_loss((const HeadProb*)(p->desc + p->head_desc_off), p->n_heads, p->stream), PACK_EDEVICE);
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    HIP_TRY(hipMemcpy(host_dst, p->loss_all, (size_t)p->K * 4, hipMemcpyDeviceToHost), PACK_EDEVICE);
    int flag = 0;
    HIP_TRY(hipMemcpy(&flag, p->err_flag, 4, hipMemcpyDeviceToHost), PACK_EDEVICE);
    if (flag) {
        HIP_TRY(hipMemset(p->err_flag, 0, 4), PACK_EDEVICE);
        if (flag & 2) return fail(PACK_EINDEX, "pack_gather_batch met a sample index outside the dataset since the last pack_read_loss");
        return fail(PACK_ELABEL, "a label outside [0, C_k) was seen since the last pack_read_loss");
    }
    return PACK_OK;
}

pack_status pack_read_weights(pack_t* p, int32_t k, float* host_dst, size_t n_floats) {
    return download(p, k, p ? p->master : nullptr, host_dst, n_floats);
}

pack_status pack_read_grads(pack_t* p, int32_t k, float* host_dst, size_t n_floats) {
    if (p && p->fused && !p->keep_grads)
        return fail(PACK_EINVAL, "plain-SGD packs apply the update where the gradient is produced and do not store it: "
                                 "call pack_keep_grads(p, 1) first");
    return download(p, k, p ? p->grad : nullptr, host_dst, n_floats);
}

pack_status pack_read_pred(pack_t* p, int32_t k, int32_t* host_dst) {
    if (!p || !host_dst) return fail(PACK_EINVAL, "null argument");
    pack_status lm = live_member(p, k);
    if (lm != PACK_OK) return lm;
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    HIP_TRY(hipMemcpy(host_dst, p->models[k].pred, (size_t)p->models[k].batch * 4, hipMemcpyDeviceToHost), PACK_EDEVICE);
    return PACK_OK;
}

pack_status pack_read_logits(pack_t* p, int32_t k, float* host_dst, size_t n_floats) {
    if (!p || !host_dst) return fail(PACK_EINVAL, "null argument");
    pack_status lm = live_member(p, k);
    if (lm != PACK_OK) return lm;
    const ModelInfo& m = p->models[k];
    if (n_floats != (size_t)m.batch * m.C) return fail(PACK_EINVAL, "n_floats must be b_k * C_k");
    HIP_TRY(hipStreamSynchronize(p->stream), PACK_EDEVICE);
    HIP_TRY(hipMemcpy(host_dst, m.tensors[m.nodes.back().out_t].act, n_floats * 4, hipMemcpyDeviceToHost), PACK_EDEVICE);
    return PACK_OK;
}

size_t pack_num_params(const pack_t* p, int32_t k) {
    if (!p || k < 0 || k >= p->K) return 0;
    return p->models[k].n_params;
}

int32_t pack_num_classes(const pack_t* p, int32_t k) {
    if (!p || k < 0 || k >= p->K) return 0;
    return p->models[k].C;
}

int32_t pack_num_launches(const pack_t* p) { return p ? (int32_t)p->plan.size() : 0; }

size_t pack_device_bytes(const pack_t* p) { return p ? p->device_bytes : 0; }

void pack_destroy(pack_t* p) {
    if (!p) return;
    (void)hipStreamSynchronize(p->stream);
    release(p);
}

}  // extern "C"
