// C ABI of the dpcert library: network description, certify orchestration, result accessors.
// The host loop mirrors the DeepPoly flow of the paper (Appendix C): layers in forward order; for
// every affine / convolution layer one backward traversal of its neurons' polyhedral expressions
// (ReLU step, contraction, ... down to the input) followed by concretisation.
#include <stdarg.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <memory>
#include <mutex>
#include <set>
#include <utility>
#include <vector>

#include <atomic>
#include <climits>

#include "common.h"
#include "conv.h"

namespace dpc {

static thread_local std::string g_error;

void ensure_dynamic_lds(const void* kernel, int bytes)
{
    static std::mutex mu;
    static std::set<std::pair<const void*, int>> done;
    int dev = 0;
    DPC_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({kernel, dev})) return;
    DPC_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    done.insert({kernel, dev});
}

void set_error(const char* fmt, ...)
{
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
}

// ---- tuning knobs: process-wide values, per-network overrides, the values in force on the calling thread ----
namespace {
struct TuneInfo { const char* name; int def; };
constexpr TuneInfo kTune[TK_COUNT] = {
    {"contract_variant", -1}, {"contract_remap", 1}, {"conv_algo", 0}, {"conv_half_tiles", 1},
    {"merge_final", 1},           // 1: output-layer bounds and margins share one traversal
    {"reuse_patch", 1},           // 1: ReuseCert keeps the stored bounds of convolution layers over their receptive fields only
    {"reuse_window", 1},          // 1: ReuseCert's steps above a convolutional front run as implicit contractions
    {"reuse_window_ck", 0}, {"reuse_window_tiles", -1}, {"chain", -1}, {"chain_rows", 64}, {"contract_split_wide", -1},
    {"contract_split", 0}, {"rows_per_wave", 0}, {"rows_stream", 1}, {"stream_wgs_per_cu", 0},
};
struct TuneTable {
    std::atomic<int> v[TK_COUNT];
    TuneTable() { for (int k = 0; k < TK_COUNT; ++k) v[k].store(kTune[k].def, std::memory_order_relaxed); }
};
TuneTable g_tune;
std::atomic<uint64_t> g_tuning_epoch{1};   // bumped by every dpc_tuning_set: captured launch sequences are keyed on it
thread_local const Tuning* t_tuning = nullptr;
constexpr int kTuneUnset = INT32_MIN;
int tune_key(const char* key)
{
    for (int k = 0; k < TK_COUNT; ++k)
        if (strcmp(key, kTune[k].name) == 0) return k;
    return -1;
}
}  // namespace

int tune(TuneKey k) { return t_tuning ? t_tuning->v[k] : g_tune.v[k].load(std::memory_order_relaxed); }
TuningScope::TuningScope(const Tuning* t) : prev_(t_tuning) { t_tuning = t; }
TuningScope::~TuningScope() { t_tuning = prev_; }

namespace {

enum Kind { AFFINE = 0, CONV = 1, RELU = 2, ADD = 3 };

// Workspace of the entry point that allocates nothing (dpc_certify_static): one array per device, held until the
// process ends.  In host code the array's name is only a handle: its device address is looked up once per device.
constexpr size_t kStaticWorkspaceBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

unsigned char* static_workspace(int device)       // `device` must be the current device
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static unsigned char* addr[kMaxDevices] = {};
    DPC_REQUIRE(device >= 0 && device < kMaxDevices, DPC_EINVAL, "device %d out of range", device);
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[device]) {
        void* p = nullptr;
        DPC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        DPC_REQUIRE(p, DPC_EHIP, "hipGetSymbolAddress returned no address for the static workspace");
        addr[device] = static_cast<unsigned char*>(p);
    }
    return addr[device];
}

struct DeviceGuard {
    int prev = -1;
    explicit DeviceGuard(int dev)
    {
        DPC_HIP(hipGetDevice(&prev));
        if (prev != dev) DPC_HIP(hipSetDevice(dev));
        else prev = -1;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

// Bump allocator over a fixed block of device memory (the library's static workspace): nothing is ever freed, the
// owner rewinds it at the start of a call.
struct Arena {
    unsigned char* base = nullptr;
    size_t size = 0, used = 0;
    void* take(size_t bytes)
    {
        const size_t at = (used + 255) & ~(size_t)255;
        DPC_REQUIRE(at + bytes <= size, DPC_EINVAL,
                    "this call needs more than the %zu MiB of the library's static workspace (network or batch too large for "
                    "the entry point that allocates nothing)", size >> 20);
        used = at + bytes;
        return base + at;
    }
};

template <class T>
struct DevBuf {
    T* p = nullptr;
    size_t count = 0;
    Arena* arena = nullptr;            // set: memory comes from the arena and is never freed here
    bool reserve(size_t n)             // true when the buffer was (re)allocated: old addresses are dead
    {
        if (n <= count) return false;
        if (arena) {
            p = static_cast<T*>(arena->take(n * sizeof(T)));
            count = n;
            return true;
        }
        release();
        DPC_HIP(hipMalloc(reinterpret_cast<void**>(&p), n * sizeof(T)));
        count = n;
        return true;
    }
    void release()
    {
        if (p && !arena) (void)hipFree(p);
        p = nullptr;
        count = 0;
    }
    ~DevBuf() { release(); }
    DevBuf() = default;
    explicit DevBuf(Arena* a) : arena(a) {}
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
};

struct Layer {
    int kind = AFFINE;
    int n_in = 0, n_out = 0;
    ConvGeom g{};                          // CONV only
    int skip = -1;                         // ADD only: layer index (0 = input) of the second operand
    bool unit_rows = false;                // ADD above a ReLU or another ADD: bounded from unit rows of its own (dW / cw hold an identity)
    bool spatial_out = false;              // neurons of this layer carry a (C,H,W) shape (stored H,W,C)
    int C = 0, H = 0, W = 0;               // that shape
    std::vector<float> hW, hb;             // host copies in the caller's layout
    // device, in the internal neuron order
    DevBuf<float> dW;                      // AFFINE: [n_out, ldw]; CONV: see conv.h
    int ldw = 0;
    DevBuf<float> dBias;                   // [n_out] per neuron
    ConvWeights cw;                        // CONV only
    // ReuseCert: [W+ | W- | b] and [W- | W+ | b], [n_out, ld_split] each, built on first use
    DevBuf<float> dSplit[2];
    int ld_split = 0;
    DevBuf<float> dDense;                  // ReuseCert, convolution as the first layer: its expanded rows [n_out, ld0]
    // split-precision experiment: bf16 terms of the transposed weights, built when the tuning key is set
    DevBuf<uint16_t> dWt;
    int wt_terms = 0;
};

}  // namespace
}  // namespace dpc

namespace dpc {
namespace {
// Device memory a certify call works in, besides the result's own arrays.
struct Workspace {
    Arena* arena = nullptr;                // set: every buffer below is carved from it
    DevBuf<float> buf[2];                  // coefficient rows, ping-pong
    DevBuf<double> cst;                    // row constants
    DevBuf<float> stage;                   // staging for layout permutations / margins
    // fused-epilogue state: packed per-(side, input, neuron) parameters of every ReLU layer (index 0:
    // the box), and the slots that collect row-constant partial sums of the fused contractions
    std::vector<std::unique_ptr<DevBuf<float>>> pk;
    DevBuf<float> pk2;                     // compact (mu, nu | lambda) of the first ReLU layer (patch-tail kernel)
    std::vector<std::unique_ptr<DevBuf<float>>> pk2v;      // the same for ReLU layers above a convolution with > 4 input channels
    DevBuf<float> rpart;                   // one constant per row from a ReLU step applied inside a convolution kernel
    DevBuf<int32_t> dflag;                 // device word of the input validation for inputs ingested by one kernel (zero between calls)
    std::vector<std::unique_ptr<DevBuf<float>>> skipbuf;   // residual networks: blocks of rows waiting on a skip connection
    DevBuf<float> part;
    int64_t part_stride = 0;
    DevBuf<float> rc_rows;                 // ReuseCert: split output/margin rows of the last step, per input
    DevBuf<float> gather;                  // ReuseCert through a convolution: gathered right operands of a chunk of positions
    uint64_t ws_epoch = 1;                 // bumped whenever a workspace buffer moves (captured graphs hold addresses)
    Workspace() = default;
    explicit Workspace(Arena* a) : arena(a), cst(a), stage(a), pk2(a), rpart(a), dflag(a), part(a), rc_rows(a), gather(a)
    {
        buf[0].arena = a;
        buf[1].arena = a;
    }
    DevBuf<float>* fresh_buf() const { return new DevBuf<float>(arena); }
};
}  // namespace
}  // namespace dpc

using namespace dpc;

struct dpc_network {
    std::vector<std::unique_ptr<Layer>> layers;
    int n0 = 0;
    bool in_spatial = false;
    int inC = 0, inH = 0, inW = 0;
    bool finalized = false;
    int device = 0;
    int live_results = 0;
    // traversal workspace, grown on demand, reused across certify calls (the entry point that allocates nothing swaps in
    // one that lives in the library's static device array for the duration of its call)
    Workspace own_ws;
    Workspace* ws = &own_ws;
    int32_t* h_flag = nullptr;             // pinned host word the input validation reports into (allocated by finalize)
    int tune_override[TK_COUNT];           // kTuneUnset: the process-wide value applies
    uint64_t tuning_epoch = 0;
    dpc_network() { for (int& v : tune_override) v = kTuneUnset; }
    Tuning tuning() const
    {
        Tuning t;
        for (int k = 0; k < TK_COUNT; ++k)
            t.v[k] = tune_override[k] != kTuneUnset ? tune_override[k] : g_tune.v[k].load(std::memory_order_relaxed);
        return t;
    }
    ~dpc_network() { if (h_flag) (void)hipHostFree(h_flag); }
    int skip_depth = 0;                    // how many skip connections span one layer at most
    static constexpr int kMaxSlots = 96;

    int size_of(int idx) const { return idx == 0 ? n0 : layers[idx - 1]->n_out; }
    int ld_of(int idx) const { return (int)round_up(size_of(idx), kLdAlign); }
    bool spatial(int idx, int* C, int* H, int* W) const
    {
        if (idx == 0) { *C = inC; *H = inH; *W = inW; return in_spatial; }
        const Layer& L = *layers[idx - 1];
        *C = L.C; *H = L.H; *W = L.W;
        return L.spatial_out;
    }
};

struct dpc_result {
    dpc_network* net = nullptr;
    int batch = 0;
    int keep_symbolic = 0;
    int certifier = DPC_DEEPPOLY;          // of the last certify call on this result
    bool has_label = false;
    std::vector<float*> l, u, lam, mu, nu;   // per layer index, device, internal order (sub-allocations)
    DevBuf<float> pool;
    DevBuf<float> margin;                    // [B, nK-1]
    DevBuf<int32_t> verdict, label;
    // kept symbolic bounds: per layer index (1..nl; nl + 1 = the property's margin rows, lower side only) the
    // input-level expressions [side][b][r] x ld0 with their constants, internal neuron orders
    std::vector<std::unique_ptr<DevBuf<float>>> sym_c;
    std::vector<std::unique_ptr<DevBuf<double>>> sym_k;
    std::vector<char> sym_have;
    dpc_profile prof{};
    // the kernel sequence of a certify call on this result, captured once and replayed on reuse
    hipGraphExec_t gexec = nullptr;
    struct GraphKey {
        int depth = 0, fuse = 0, has_label = 0;
        uint64_t tuning_epoch = 0, ws_epoch = 0;
        bool operator==(const GraphKey& o) const
        {
            return depth == o.depth && fuse == o.fuse && has_label == o.has_label && tuning_epoch == o.tuning_epoch &&
                   ws_epoch == o.ws_epoch;
        }
    } gkey;
    dpc_profile gprof{};                   // launch and flop counters of the captured sequence
    dpc_result() = default;
    explicit dpc_result(Arena* a) : pool(a), margin(a), verdict(a), label(a) {}
    ~dpc_result() { if (gexec) (void)hipGraphExecDestroy(gexec); }
};

namespace {

// Per-kernel-class timing with HIP events on the launch stream.  One event is recorded whenever the
// class of the next launch differs from the class of the previous one, so a run of back-to-back
// launches of one class costs two events, not two per launch.
struct Prof {
    bool on = false;
    hipStream_t s = nullptr;
    struct Seg { int cls; hipEvent_t a, b; };
    std::vector<Seg> segs;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    int cur = -1;
    hipEvent_t get()
    {
        if (used == pool.size()) {
            hipEvent_t e;
            DPC_HIP(hipEventCreate(&e));
            pool.push_back(e);
        }
        return pool[used++];
    }
    void begin(int cls)
    {
        if (!on || cls == cur) return;
        hipEvent_t e = get();
        DPC_HIP(hipEventRecord(e, s));
        if (cur >= 0) segs.back().b = e;
        segs.push_back(Seg{cls, e, nullptr});
        cur = cls;
    }
    void end() {}
    void finish()
    {
        if (!on || cur < 0) return;
        hipEvent_t e = get();
        DPC_HIP(hipEventRecord(e, s));
        segs.back().b = e;
        cur = -1;
    }
    ~Prof() { for (auto e : pool) (void)hipEventDestroy(e); }
};
enum { P_CONTRACT = 0, P_RELAX = 1, P_CONC = 2, P_OTHER = 3, P_CHAIN = 4 };

// Shape of the coefficient rows during a traversal: dense over a whole layer, or patch form
// (rows of a convolution layer: a small window of the current layer, see conv.h).
struct Form {
    bool patch = false;
    PatchGeom pg{};
    int ld = 0;
};

Form start_form(const dpc_network* net, int at, const Layer* own)
{
    Form f;
    if (own && (own->kind == CONV || (own->kind == ADD && own->spatial_out))) {     // (ADD: 1x1 identity cores over its operand)
        const ConvGeom& g = own->g;
        f.patch = true;
        f.pg = PatchGeom{g.Wo, g.Co, g.kh, g.kw, g.Ci, g.stride, g.pad, g.H, g.W};
        f.ld = own->cw.ld_core;
    } else {
        f.ld = net->ld_of(at);
    }
    return f;
}

// Form after a traverse iteration through convolution layer g (patch form only).
Form through_conv(const Form& f, const ConvGeom& g)
{
    Form o = f;
    o.pg.ph = (f.pg.ph - 1) * g.stride + g.kh;
    o.pg.pw = (f.pg.pw - 1) * g.stride + g.kw;
    o.pg.C = g.Ci;
    o.pg.S = f.pg.S * g.stride;
    o.pg.P = f.pg.P * g.stride + g.pad;
    o.pg.gh = g.H;
    o.pg.gw = g.W;
    o.ld = (int)round_up(o.pg.elems(), 4);
    return o;
}

// Largest rows x leading-dimension product any traversal of this network needs, in floats.
size_t workspace_floats(const dpc_network* net, int B, bool with_margin)
{
    size_t need = 1;
    const int nl = (int)net->layers.size();
    for (int i = 1; i <= nl; ++i) {
        if (net->layers[i - 1]->kind == RELU) continue;
        // an Add layer is bounded through the rows of the layer below it (plus a unit block on the skip operand)
        const int top = (net->layers[i - 1]->kind == ADD && !net->layers[i - 1]->unit_rows) ? i - 1 : i;
        const Layer& own = *net->layers[top - 1];
        const size_t rows = 2 * (size_t)B * own.n_out;
        Form f = start_form(net, top - 1, &own);
        need = std::max(need, rows * f.ld);
        for (int at = top - 1; at > 0; --at) {
            const Layer& L = *net->layers[at - 1];
            if (L.kind == CONV && f.patch) f = through_conv(f, L.g);
            else if (L.kind == AFFINE || L.kind == CONV) f.ld = net->ld_of(at - 1);
            need = std::max(need, rows * f.ld);
        }
    }
    if (with_margin) {
        const size_t rows = 2 * (size_t)B * std::max<size_t>(2 * (size_t)net->layers[nl - 1]->n_out - 1, 32);
        for (int j = 0; j < nl; ++j) need = std::max(need, rows * net->ld_of(j));
    }
    return need;
}

// One backward traversal (backsubs_lower and backsubs_upper of R expressions per input) starting
// from expressions over layer index `at`: either the shared weight rows of layer `own`, or per-input
// rows already in net->ws->buf[0] (own == NULL).
struct Pass {
    dpc_network* net;
    dpc_result* res;
    const dpc_options* opt;
    hipStream_t s;
    Prof* prof;
    int B;
    int maxd;             // traversal limit of this pass (-1: to the input)
    bool fuse;            // the call filled the packed ReLU parameters (pk, pk2, pk2v) of every layer: only then may a
                          // kernel that applies a ReLU step from them be chosen (an earlier call's are stale)
    // Work that can ride on the pass's last kernel when that kernel is the fold of the partial sums (no launch of its own):
    // the parameters of the ReLU layer above the bounded layer, or the split of the merged last pass.
    struct NextRelu { float *lam, *mu, *nu, *rl, *ru; const float* bias; int n, ld; float *pk, *pk2; };
    struct FinalSplit { int nK, Rs; float *l, *u, *margin; int32_t* verdict; };
    const NextRelu* next = nullptr;
    const FinalSplit* fin = nullptr;
    bool rider_done = false;      // set by the pass when it did that work
};

// A block of the expression that waits on a skip connection until the traversal reaches the layer it is over
// (residual networks: the expression then has terms on two layers at once).
struct Waiting {
    int target;            // layer index the block is over
    int kind;              // 0: rows of its own (src = a skip buffer), 1: the bounded layer's shared rows / cores, 2: unit block
    const float* src;
    int ld;
    int slot;              // kind 0: 0 when src is a buffer of the pool (returned when the block is merged), else -1
    bool patch;
    int ph, pw, S, P;      // patch geometry of the block when it was set aside
};

// diag_target >= 0: the expressions are those of an Add layer's neurons, i.e. the rows of `own` (the layer below the Add
// layer) plus coefficient 1 on the same neuron of layer diag_target.
void run_pass(Pass& P, int at, int nsides, int R, const Layer* own, float* out_l, float* out_u, int sym_idx,      // sym_idx >= 0: keep the input-level expressions there
              double useful = 1.0,       // fraction of the rows whose bounds are used (flop accounting only)
              int diag_target = -1, int depth0 = 0)    // depth0: traverse iterations the starting rows already stand for
{
    dpc_network* net = P.net;
    dpc_result* res = P.res;
    const int B = P.B;
    const int maxd = P.maxd;
    const bool keep_sym = sym_idx >= 0;
    float* cur = net->ws->buf[0].p;
    float* nxt = net->ws->buf[1].p;
    double* cst = net->ws->cst.p;
    Form f = start_form(net, at, own);
    // rows not yet per-input: the layer's own weight rows (dense) or kernel cores (patch form)
    const float* shared = own ? (f.patch ? own->cw.core : own->dW.p) : nullptr;
    const int ld_shared = own ? (f.patch ? own->cw.ld_core : own->ldw) : 0;
    const float* cst_init = own ? (f.patch ? own->cw.bias_c : own->dBias.p) : nullptr;
    bool bias_folded = false;
    bool bias_below_add = false;           // the ReLU step above an Add layer has already folded the bias of the layer below the Add
    int depth = depth0;
    const int64_t M = (int64_t)nsides * B * R;
    bool fused_relu = false;
    int slots = 0;                 // row-constant partial-sum slots written by fused epilogues so far
    bool concretised = false;      // the last contraction already reduced the rows against the box
    const int split = contract_split_terms();       // > 0: contractions on the bf16 MFMA units, every step its own kernel
    const bool may_fuse = P.fuse && maxd < 0 && !keep_sym && R >= 32 && net->ws->part.p && M <= net->ws->part_stride;

    std::vector<Waiting> waiting;
    // Row buffers: cur / nxt plus the pool of skip buffers (all of one size).  When the rows cross an Add layer they are
    // not copied: the buffer they sit in is kept for the waiting block and, once the next contraction has read it, a
    // buffer from the pool takes its place in the cur / nxt pair (nothing writes the rows in place before that
    // contraction: the layer below an Add layer is affine or convolution).
    std::vector<float*> pool;
    for (int k = (int)net->ws->skipbuf.size() - 1; k >= 0; --k) pool.push_back(net->ws->skipbuf[k]->p);
    float* held = nullptr;         // buffer of the rows set aside at the last Add layer while it is still `cur`
    float* spare = nullptr;        // the pool buffer that replaces it
    auto after_swap = [&]() {
        if (held && nxt == held) { nxt = spare; held = nullptr; spare = nullptr; }
    };
    if (diag_target >= 0) waiting.push_back(Waiting{diag_target, 2, nullptr, 0, -1, f.patch, 1, 1, 1, 0});
    auto blocked = [&](int idx) {
        for (const Waiting& w : waiting)
            if (w.target == idx) return true;
        return false;
    };

    // Fully-connected layers all the way down: the whole traversal in one kernel, rows resident in LDS.
    if (split == 0 && waiting.empty() && may_fuse && own && own->kind == AFFINE && !f.patch && nsides == 2 && at >= 1 && net->layers[at - 1]->kind == RELU &&
        net->ws->pk[at] && net->ws->pk[at]->p) {
        ChainStepDesc steps[16];
        int ns = 0;
        bool ok = true;
        double flop = 0.0;
        for (int j = at - 1; ok; j -= 2) {          // j: 1-based index of the affine layer the step crosses
            if (j < 1 || ns >= 16) { ok = false; break; }
            const Layer& L = *net->layers[j - 1];
            const int below = j - 1;
            if (L.kind != AFFINE || !net->ws->pk[below] || !net->ws->pk[below]->p) { ok = false; break; }
            if (below > 0 && net->layers[below - 1]->kind != RELU) { ok = false; break; }
            steps[ns++] = ChainStepDesc{L.dW.p, net->ws->pk[below]->p, L.n_out, L.ldw, net->ld_of(below), below > 0 ? 1 : 0};
            flop += 2.0 * (double)M * L.n_out * L.n_in;
            if (below == 0) break;
        }
        if (ok) {
            ChainDesc d{own->dW.p, own->dBias.p, net->ws->pk[at]->p, own->ldw, net->ld_of(at), net->ld_of(at), R, B, ns, steps,
                        out_l, out_u};
            P.prof->begin(P_CHAIN);
            const bool done = launch_chain(d, P.s);
            P.prof->end();
            if (done) {
                res->prof.chain_flop += useful * flop;
                res->prof.chain_launches++;
                return;
            }
        }
    }

    auto relax = [&](const float* la, const float* m, const float* v, const Layer* bias_of) {
        const int n_at = net->size_of(at);
        P.prof->begin(P_RELAX);
        if (f.patch)
            launch_relax_step_patch(cur, f.ld, cst, nsides, B, R, f.pg, la, m, v, bias_of ? bias_of->cw.bias_c : nullptr,
                                    shared, ld_shared, cst_init, P.s);
        else
            launch_relax_step(cur, f.ld, cst, nsides, B, R, n_at, la, m, v, bias_of ? bias_of->dBias.p : nullptr,
                              shared, ld_shared, shared ? cst_init : nullptr, P.s);
        P.prof->end();
        res->prof.relax_launches++;
        res->prof.relax_bytes += (double)M * (f.patch ? f.pg.elems() : n_at) * (shared ? 4.0 : 8.0);
        shared = nullptr;
    };

    // blocks that waited for layer idx are added to the rows (which must be per-input rows by then)
    auto merge_at = [&](int idx) {
        for (size_t k = 0; k < waiting.size();) {
            if (waiting[k].target != idx) { ++k; continue; }
            const Waiting w = waiting[k];
            if (shared) relax(nullptr, nullptr, nullptr, nullptr);
            P.prof->begin(P_RELAX);
            if (f.patch) {
                DPC_REQUIRE(w.patch && w.S == f.pg.S && f.pg.P >= w.P, DPC_EUNSUPPORTED,
                            "a skip connection across layers that change the stride is not supported");
                launch_merge_block(cur, f.ld, M, R, f.pg.rows_C, f.pg.ph, f.pg.pw, f.pg.C, w.kind, w.src, w.ld, w.ph, w.pw,
                                   f.pg.P - w.P, P.s);
            } else {
                DPC_REQUIRE(!w.patch, DPC_EUNSUPPORTED, "patch-form block waiting for dense rows");
                launch_merge_block(cur, f.ld, M, R, R, 1, 1, net->size_of(idx), w.kind, w.src, w.ld, 1, 1, 0, P.s);
            }
            P.prof->end();
            res->prof.relax_launches++;
            if (w.slot >= 0) {
                // back to the pool -- unless the block's buffer is still one of the pair (no contraction since the Add
                // layer): then the spare one goes back instead
                if (w.src == held) { pool.push_back(spare); held = nullptr; spare = nullptr; }
                else pool.push_back(const_cast<float*>(w.src));
            }
            waiting.erase(waiting.begin() + k);
        }
    };

    while (at > 0 && (maxd < 0 || depth < maxd)) {
        merge_at(at);
        const Layer& L = *net->layers[at - 1];
        if (L.kind == ADD) {
            // neurons of this layer = layer below + layer L.skip: the rows go on through the layer below, a copy waits
            Waiting w{L.skip, 0, nullptr, 0, -1, f.patch, f.pg.ph, f.pg.pw, f.pg.S, f.pg.P};
            if (shared) {
                w.kind = 1; w.src = shared; w.ld = ld_shared;
            } else {
                DPC_REQUIRE(!pool.empty(), DPC_EUNSUPPORTED, "skip connections nested deeper than the workspace allows");
                w.slot = 0;
                w.ld = f.ld;
                const int kind_below = net->layers[at - 2]->kind;
                if (held || blocked(at - 1) || L.skip == at - 1 || (kind_below != AFFINE && kind_below != CONV)) {
                    // another block joins the rows at the layer below (in place), the next step rewrites the rows in place
                    // (a ReLU layer below, directly or under another Add layer), or the previous Add layer's buffer is still
                    // one of the pair: a copy waits
                    float* dst = pool.back();
                    pool.pop_back();
                    DPC_HIP(hipMemcpyAsync(dst, cur, (size_t)M * f.ld * sizeof(float), hipMemcpyDeviceToDevice, P.s));
                    w.src = dst;
                } else {
                    held = cur;
                    spare = pool.back();
                    pool.pop_back();
                    w.src = cur;
                }
            }
            waiting.push_back(w);
            bias_folded = bias_below_add;
            bias_below_add = false;
            fused_relu = false;
            --at;
            ++depth;
            continue;
        }
        if (waiting.empty() && L.kind == RELU && at == 2 && f.patch && nsides == 2 && P.fuse && maxd < 0 && !keep_sym && net->ws->pk2.p &&
            net->layers[0]->kind == CONV && (shared != nullptr || bias_folded || depth > 0)) {
            // patch rows over the first ReLU layer: ReLU step, first layer and concretisation in one kernel
            const Layer& first = *net->layers[0];
            PatchTail pt{shared ? shared : cur, shared ? ld_shared : f.ld, shared ? 1 : 0, cst, cst_init, R, B, &f.pg, &first.g,
                         net->ws->pk2.p, net->ld_of(2), first.cw.bias_c, first.cw.taps, res->l[0], res->u[0], out_l, out_u};
            P.prof->begin(P_CONTRACT);
            const bool done = launch_patch_tail(pt, P.s);
            P.prof->end();
            if (done) {
                res->prof.contract_flop += useful * 2.0 * (double)M * f.pg.ph * f.pg.pw * first.g.Co * first.g.Ci * first.g.kh * first.g.kw;
                res->prof.contract_launches++;
                return;
            }
        }
        if (waiting.empty() && L.kind == RELU && at == 2 && !f.patch && !shared && P.fuse && maxd < 0 && !keep_sym && net->ws->pk2.p &&
            net->layers[0]->kind == CONV && net->ws->part.p && M <= net->ws->part_stride && slots < dpc_network::kMaxSlots) {
            // dense rows over the first ReLU layer: its step is applied while the first layer's transposed convolution
            // loads the rows (no pass of its own over them); the constants it adds arrive in slots
            const Layer& first = *net->layers[0];
            const ReluOnLoad rl{net->ws->pk2.p, net->ld_of(2), first.cw.bias_c, net->ws->part.p + (size_t)slots * net->ws->part_stride,
                                net->ws->part_stride, dpc_network::kMaxSlots - slots, R, B, nullptr, 0};
            int used = 0;
            P.prof->begin(P_CONTRACT);
            const bool done = launch_conv_transpose_fast(cur, M, f.ld, first.g.Ho, first.g.Wo, first.g, first.cw, nxt, net->ld_of(0),
                                                         first.g.H, first.g.W, first.g.pad, P.s, &rl, &used);
            P.prof->end();
            if (done) {
                res->prof.contract_flop += useful * 2.0 * (double)M * first.g.Ho * first.g.Wo * first.g.Co * first.g.Ci * first.g.kh * first.g.kw;
                res->prof.contract_launches++;
                slots += used;
                std::swap(cur, nxt);
                after_swap();
                f.ld = net->ld_of(0);
                at = 0;
                depth += 2;
                break;
            }
        }
        if (L.kind == RELU && at >= 3 && (!shared || cst_init) && net->layers[at - 2]->kind == CONV && net->layers[at - 2]->g.Ci > 4 && P.fuse &&
            (maxd < 0 || depth + 2 <= maxd) && (int)net->ws->pk2v.size() > at && net->ws->pk2v[at] && net->ws->pk2v[at]->p && net->ws->rpart.p &&
            (size_t)M <= net->ws->rpart.count && !blocked(at - 1)) {
            // ReLU step applied while the transposed convolution below stages the rows (no pass of its own over them); the
            // constants it adds come back in one slot and are folded into the row constants right away
            const Layer& cv = *net->layers[at - 2];
            // rows still shared by all inputs (first step of a pass): patch cores repeat every rows_C rows, weight rows every R
            const int in_mod = shared ? (f.patch ? f.pg.rows_C : R) : 0;
            const float* src = shared ? shared : cur;
            const int ld_src = shared ? ld_shared : f.ld;
            const ReluOnLoad rl{net->ws->pk2v[at]->p, net->ld_of(at), cv.cw.bias_c, net->ws->rpart.p, (int64_t)net->ws->rpart.count, 1, R, B,
                                f.patch ? &f.pg : nullptr, in_mod};
            int used = 0;
            bool done;
            Form o = f;
            P.prof->begin(P_CONTRACT);
            if (f.patch) {
                o = through_conv(f, cv.g);
                done = launch_conv_transpose_fast(src, M, ld_src, f.pg.ph, f.pg.pw, cv.g, cv.cw, nxt, o.ld, o.pg.ph, o.pg.pw, 0, P.s, &rl, &used);
            } else {
                o.ld = net->ld_of(at - 2);
                done = launch_conv_transpose_fast(src, M, ld_src, cv.g.Ho, cv.g.Wo, cv.g, cv.cw, nxt, o.ld, cv.g.H, cv.g.W, cv.g.pad, P.s, &rl,
                                                  &used);
            }
            if (done) launch_fold_slots(cst, net->ws->rpart.p, used, (int64_t)net->ws->rpart.count, M, P.s, shared ? cst_init : nullptr, in_mod);
            P.prof->end();
            if (done) {
                const double pos = f.patch ? (double)f.pg.ph * f.pg.pw : (double)cv.g.Ho * cv.g.Wo;
                res->prof.contract_flop += useful * 2.0 * (double)M * pos * cv.g.Co * cv.g.Ci * cv.g.kh * cv.g.kw;
                res->prof.contract_launches++;
                std::swap(cur, nxt);
                after_swap();
                f = o;
                shared = nullptr;
                bias_folded = false;
                fused_relu = false;
                at -= 2;
                depth += 2;
                continue;
            }
        }
        if (L.kind == RELU) {
            const Layer& below = *net->layers[at - 2];
            // the bias of the layer below is folded in the same pass unless a block still has to join the rows there
            const bool fold = (maxd < 0 || depth + 2 <= maxd) && !blocked(at - 1);
            // an Add layer passes the coefficients on unchanged to the layer below it, whose bias can be folded in this
            // same pass (full traversals only, and only if no block joins the rows between here and there)
            const Layer* bias_src = &below;
            bias_below_add = false;
            if (fold && below.kind == ADD && maxd < 0 && at >= 3 && !blocked(at - 2) &&
                (net->layers[at - 3]->kind == AFFINE || net->layers[at - 3]->kind == CONV)) {
                bias_src = net->layers[at - 3].get();
                bias_below_add = true;
            }
            relax(res->lam[at], res->mu[at], res->nu[at], fold ? bias_src : nullptr);
            bias_folded = fold;
        } else {
            if (!bias_folded) relax(nullptr, nullptr, nullptr, &L);   // affine layer entered without a ReLU step above it
            const int n_at = net->size_of(at), n_prev = net->size_of(at - 1);
            P.prof->begin(P_CONTRACT);
            if (L.kind == AFFINE) {
                DPC_REQUIRE(!f.patch, DPC_EUNSUPPORTED, "patch-form rows cannot cross a fully-connected layer");
                const int ld_prev = net->ld_of(at - 1);
                // The step that follows (ReLU step of the layer below, or the concretisation at the input)
                // runs in the contraction's epilogue when its packed parameters exist.
                const int below = at - 1;
                const bool to_input = below == 0 && !keep_sym && !blocked(0);
                const bool to_relu = below > 0 && net->layers[below - 1]->kind == RELU && !blocked(below) && !blocked(below - 1);
                int used = -1;
                fused_relu = false;
                if (may_fuse && (to_input || to_relu) && net->ws->pk[below] && net->ws->pk[below]->p) {
                    ContractEpilogue e{net->ws->pk[below]->p, ld_prev, R, nsides * B,
                                       net->ws->part.p + (size_t)slots * net->ws->part_stride, net->ws->part_stride,
                                       dpc_network::kMaxSlots - slots, to_input ? 0 : 1};
                    used = (split > 0 && L.wt_terms == split && L.dWt.p)
                               ? launch_contract_split_fused(cur, M, n_at, f.ld, L.dWt.p, split, n_prev, nxt, ld_prev, e, P.s)
                               : launch_contract_fused(cur, M, n_at, f.ld, L.dW.p, n_prev, L.ldw, nxt, ld_prev, e, P.s);
                }
                if (used >= 0) {
                    slots += used;
                    if (to_input) concretised = true;
                    else { --at; ++depth; fused_relu = true; }       // the ReLU layer below has been replaced too
                } else if (split > 0 && L.wt_terms == split && L.dWt.p) {
                    launch_contract_split(cur, M, n_at, f.ld, L.dWt.p, split, n_prev, nxt, ld_prev, P.s);
                } else {
                    launch_contract(cur, M, n_at, f.ld, L.dW.p, n_prev, L.ldw, nxt, ld_prev, P.s);
                }
                res->prof.contract_flop += useful * 2.0 * (double)M * n_at * n_prev;
                f.ld = ld_prev;
            } else if (f.patch) {
                fused_relu = false;
                const Form o = through_conv(f, L.g);
                res->prof.contract_flop += launch_conv_transpose_rows(cur, M, f.ld, f.pg.ph, f.pg.pw, L.g, L.cw, nxt, o.ld,
                                                                      o.pg.ph, o.pg.pw, 0, P.s);
                f = o;
            } else {
                fused_relu = false;
                const int ld_prev = net->ld_of(at - 1);
                res->prof.contract_flop += useful * launch_conv_transpose_rows(cur, M, f.ld, L.g.Ho, L.g.Wo, L.g, L.cw, nxt, ld_prev,
                                                                      L.g.H, L.g.W, L.g.pad, P.s);
                f.ld = ld_prev;
            }
            P.prof->end();
            res->prof.contract_launches++;
            std::swap(cur, nxt);
            after_swap();
            bias_folded = fused_relu;
        }
        --at;
        ++depth;
    }

    merge_at(at);
    if (!waiting.empty()) {
        // the depth limit was reached while blocks still wait on skip connections: simplify_* maps over the terms of
        // every layer the expression holds, so each waiting block is concretised against its own layer's stored bounds
        DPC_REQUIRE(!keep_sym, DPC_EUNSUPPORTED, "symbolic bounds need a full traversal");
        if (shared) relax(nullptr, nullptr, nullptr, nullptr);        // constants live in cst from here on
        while (!waiting.empty()) {
            const int tgt = waiting.front().target;
            std::vector<Waiting> grp;
            for (size_t k = 0; k < waiting.size();)
                if (waiting[k].target == tgt) { grp.push_back(waiting[k]); waiting.erase(waiting.begin() + k); }
                else ++k;
            int gc = 0, gh = 0, gw = 0;
            const bool sp = net->spatial(tgt, &gc, &gh, &gw);
            Waiting w = grp[0];
            if (grp.size() > 1) {
                // blocks over one layer are one block of the expression (the sign split is taken on their sum): they are
                // summed in the free row buffer, in the smallest patch that holds them all
                int Pm = 0, phm = 1, pwm = 1;
                for (const Waiting& x : grp) {
                    DPC_REQUIRE(x.patch == w.patch && (!x.patch || x.S == w.S), DPC_EUNSUPPORTED, "waiting blocks of different forms");
                    Pm = std::max(Pm, x.P);
                }
                for (const Waiting& x : grp) { phm = std::max(phm, Pm - x.P + x.ph); pwm = std::max(pwm, Pm - x.P + x.pw); }
                const int n_t = net->size_of(tgt);
                const int ldm = w.patch ? (int)round_up((int64_t)phm * pwm * gc, 4) : net->ld_of(tgt);
                DPC_REQUIRE((size_t)M * ldm <= std::min(net->ws->buf[0].count, net->ws->buf[1].count), DPC_EUNSUPPORTED,
                            "waiting blocks do not fit the workspace");
                P.prof->begin(P_RELAX);
                launch_fill_zero(nxt, M * ldm, P.s);
                for (const Waiting& x : grp) {
                    if (w.patch)
                        launch_merge_block(nxt, ldm, M, R, f.pg.rows_C, phm, pwm, gc, x.kind, x.src, x.ld, x.ph, x.pw, Pm - x.P, P.s);
                    else
                        launch_merge_block(nxt, ldm, M, R, R, 1, 1, n_t, x.kind, x.src, x.ld, 1, 1, 0, P.s);
                }
                P.prof->end();
                res->prof.relax_launches += 1 + (int)grp.size();
                w.kind = 0; w.src = nxt; w.ld = ldm; w.ph = phm; w.pw = pwm; w.P = Pm;
            }
            DPC_REQUIRE(!w.patch || sp, DPC_EUNSUPPORTED, "patch-form block over a layer without a shape");
            P.prof->begin(P_CONC);
            launch_block_bound(cst, M, R, f.patch ? f.pg.rows_C : R, f.patch ? f.pg.rows_W : 1, B, nsides, net->size_of(tgt), w.kind,
                               w.src, w.ld, res->l[tgt], res->u[tgt], w.patch ? 1 : 0, w.ph, w.pw, gc, w.S, w.P, gh, gw, P.s);
            P.prof->end();
            res->prof.concretise_launches++;
        }
        waiting.clear();
    }
    const int n_at = net->size_of(at);
    if (keep_sym) {
        DPC_REQUIRE(at == 0, DPC_EUNSUPPORTED, "symbolic bounds are kept at the input only");
        float* dc = res->sym_c[sym_idx]->p;
        double* dk = res->sym_k[sym_idx]->p;
        const int ld0 = net->ld_of(0);
        if (f.patch) {
            // rows of a convolution layer reach the input as patches: written out as dense rows over the input
            launch_fill_zero(dc, M * ld0, P.s);
            launch_expand_patch_rows(shared ? shared : cur, shared ? ld_shared : f.ld, shared ? f.pg.rows_C : 0, cst, cst_init, M, R,
                                     f.pg.rows_C, f.pg.rows_W, f.pg.ph, f.pg.pw, f.pg.C, f.pg.S, f.pg.P, f.pg.gh, f.pg.gw, dc, ld0, dk, P.s);
        } else if (!shared) {
            DPC_HIP(hipMemcpyAsync(dc, cur, (size_t)M * f.ld * sizeof(float), hipMemcpyDeviceToDevice, P.s));
            DPC_HIP(hipMemcpyAsync(dk, cst, (size_t)M * sizeof(double), hipMemcpyDeviceToDevice, P.s));
        } else {
            // first layer: the expression is the weight row itself for every input and side
            launch_relax_step(dc, f.ld, dk, nsides, B, R, n_at, nullptr, nullptr, nullptr,
                              nullptr, shared, ld_shared, cst_init, P.s);
        }
        res->sym_have[sym_idx] = 1;
    }
    P.prof->begin(P_CONC);
    if (concretised) {
        if (P.next && nsides == 2 && R == P.next->n) {
            launch_finalize_relax_pack(cst, net->ws->part.p, slots, net->ws->part_stride, out_l, out_u, P.next->lam, P.next->mu, P.next->nu,
                                       P.next->rl, P.next->ru, P.next->bias, B, R, P.next->ld, P.next->pk, P.next->pk2, P.s);
            P.rider_done = true;
        } else if (P.fin && nsides == 2 && R == P.fin->Rs &&
                   launch_finalize_split_final(cst, net->ws->part.p, slots, net->ws->part_stride, B, P.fin->nK, R, P.fin->l, P.fin->u,
                                               P.fin->margin, P.fin->verdict, P.s)) {
            P.rider_done = true;
        } else {
            launch_finalize_bounds(cst, net->ws->part.p, slots, net->ws->part_stride, nsides, B, R, out_l, out_u, P.s);
        }
    } else if (f.patch) {
        launch_concretise_patch(cur, f.ld, cst, nsides, B, R, f.pg, res->l[at], res->u[at], out_l, out_u,
                                shared, ld_shared, cst_init, P.s);
        res->prof.concretise_bytes += (double)M * f.pg.elems() * 4.0;
    } else {
        launch_concretise(cur, f.ld, cst, nsides, B, R, n_at, res->l[at], res->u[at], out_l, out_u,
                          shared, ld_shared, shared ? cst_init : nullptr, P.s, net->ws->part.p, slots, net->ws->part_stride);
        // rows still shared by all inputs (a first layer) are one weight matrix, read once
        res->prof.concretise_bytes += (double)(shared ? R : M) * n_at * 4.0;
    }
    P.prof->end();
    res->prof.concretise_launches++;
}

void validate_chain(dpc_network* net)
{
    DPC_REQUIRE(!net->layers.empty(), DPC_EINVAL, "network has no layers");
    DPC_REQUIRE(net->layers[0]->kind != RELU, DPC_EUNSUPPORTED, "ReLU cannot be the first layer");
    DPC_REQUIRE(net->layers.back()->kind != RELU, DPC_EUNSUPPORTED, "ReLU after the last affine layer is not supported");
    for (size_t i = 1; i < net->layers.size(); ++i) {
        DPC_REQUIRE(!(net->layers[i]->kind == RELU && net->layers[i - 1]->kind == RELU), DPC_EUNSUPPORTED,
                    "two ReLU layers in a row");
        DPC_REQUIRE(net->layers[i]->n_in == net->layers[i - 1]->n_out, DPC_EINVAL,
                    "layer %zu expects %d inputs but the previous layer has %d neurons", i + 1,
                    net->layers[i]->n_in, net->layers[i - 1]->n_out);
    }
}

bool all_finite(const float* p, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (!std::isfinite(p[i])) return false;
    return true;
}

template <class F>
dpc_status guarded(F&& f)
{
    try {
        f();
        return DPC_OK;
    } catch (const Fail& e) {
        return e.code;
    } catch (const std::bad_alloc&) {
        set_error("host allocation failed");
        return DPC_ENOMEM;
    } catch (...) {
        set_error("unexpected internal error");
        return DPC_EHIP;
    }
}

}  // namespace

extern "C" {

const char* dpc_last_error(void) { return g_error.c_str(); }
const char* dpc_version(void) { return "dpcert 0.1 (gfx950)"; }

dpc_status dpc_network_create(dpc_network** out)
{
    return guarded([&] {
        DPC_REQUIRE(out, DPC_EINVAL, "dpc_network_create: out is NULL");
        *out = new dpc_network();
    });
}

dpc_status dpc_network_add_affine(dpc_network* net, int32_t out_dim, int32_t in_dim, const float* W, const float* b)
{
    return guarded([&] {
        DPC_REQUIRE(net && W && b, DPC_EINVAL, "dpc_network_add_affine: NULL argument");
        DPC_REQUIRE(!net->finalized, DPC_ESTATE, "network already finalized");
        DPC_REQUIRE(out_dim >= 1 && in_dim >= 1 && out_dim <= (1 << 24) && in_dim <= (1 << 24), DPC_EINVAL,
                    "dpc_network_add_affine: bad dimensions %d x %d", out_dim, in_dim);
        const int prev = net->layers.empty() ? 0 : net->layers.back()->n_out;
        DPC_REQUIRE(net->layers.empty() || prev == in_dim, DPC_EINVAL,
                    "dpc_network_add_affine: in_dim %d does not match previous layer size %d", in_dim, prev);
        DPC_REQUIRE(all_finite(W, (size_t)out_dim * in_dim) && all_finite(b, out_dim), DPC_EINVAL,
                    "dpc_network_add_affine: non-finite weight or bias");
        auto L = std::make_unique<Layer>();
        L->kind = AFFINE;
        L->n_in = in_dim;
        L->n_out = out_dim;
        L->hW.assign(W, W + (size_t)out_dim * in_dim);
        L->hb.assign(b, b + out_dim);
        if (net->layers.empty()) net->n0 = in_dim;
        net->layers.push_back(std::move(L));
    });
}

dpc_status dpc_network_add_conv2d(dpc_network* net, int32_t Ci, int32_t H, int32_t W, int32_t Co, int32_t kh,
                                  int32_t kw, int32_t stride, int32_t pad, const float* K, const float* b)
{
    return guarded([&] {
        DPC_REQUIRE(net && K && b, DPC_EINVAL, "dpc_network_add_conv2d: NULL argument");
        DPC_REQUIRE(!net->finalized, DPC_ESTATE, "network already finalized");
        DPC_REQUIRE(Ci >= 1 && H >= 1 && W >= 1 && Co >= 1 && kh >= 1 && kw >= 1 && stride >= 1 && pad >= 0 &&
                        pad < kh && pad < kw && H + 2 * pad >= kh && W + 2 * pad >= kw,
                    DPC_EINVAL, "dpc_network_add_conv2d: bad geometry");
        DPC_REQUIRE((int64_t)Ci * H * W <= (1 << 24), DPC_EINVAL, "dpc_network_add_conv2d: input too large");
        const int n_in = Ci * H * W;
        const int prev = net->layers.empty() ? 0 : net->layers.back()->n_out;
        DPC_REQUIRE(net->layers.empty() || prev == n_in, DPC_EINVAL,
                    "dpc_network_add_conv2d: Ci*H*W = %d does not match previous layer size %d", n_in, prev);
        if (!net->layers.empty()) {
            const Layer& pl = *net->layers.back();
            DPC_REQUIRE(!pl.spatial_out || (pl.C == Ci && pl.H == H && pl.W == W), DPC_EINVAL,
                        "dpc_network_add_conv2d: input shape (%d,%d,%d) differs from the previous layer's (%d,%d,%d)",
                        Ci, H, W, pl.C, pl.H, pl.W);
            DPC_REQUIRE(pl.spatial_out, DPC_EUNSUPPORTED, "convolution after a fully-connected layer is not supported");
        }
        const size_t nk = (size_t)Co * Ci * kh * kw;
        DPC_REQUIRE(all_finite(K, nk) && all_finite(b, Co), DPC_EINVAL, "dpc_network_add_conv2d: non-finite weight or bias");
        auto L = std::make_unique<Layer>();
        L->kind = CONV;
        L->g = ConvGeom{Ci, H, W, Co, kh, kw, stride, pad, (H + 2 * pad - kh) / stride + 1, (W + 2 * pad - kw) / stride + 1};
        DPC_REQUIRE((int64_t)Co * L->g.Ho * L->g.Wo <= (1 << 24), DPC_EINVAL, "dpc_network_add_conv2d: output too large");
        L->n_in = n_in;
        L->n_out = Co * L->g.Ho * L->g.Wo;
        L->spatial_out = true;
        L->C = Co; L->H = L->g.Ho; L->W = L->g.Wo;
        L->hW.assign(K, K + nk);
        L->hb.assign(b, b + Co);
        if (net->layers.empty()) {
            net->n0 = n_in;
            net->in_spatial = true;
            net->inC = Ci; net->inH = H; net->inW = W;
        }
        net->layers.push_back(std::move(L));
    });
}

dpc_status dpc_network_add_relu(dpc_network* net)
{
    return guarded([&] {
        DPC_REQUIRE(net, DPC_EINVAL, "dpc_network_add_relu: NULL network");
        DPC_REQUIRE(!net->finalized, DPC_ESTATE, "network already finalized");
        DPC_REQUIRE(!net->layers.empty(), DPC_EUNSUPPORTED, "ReLU cannot be the first layer");
        const Layer& pl = *net->layers.back();
        DPC_REQUIRE(pl.kind != RELU, DPC_EUNSUPPORTED, "two ReLU layers in a row");
        auto L = std::make_unique<Layer>();
        L->kind = RELU;
        L->n_in = L->n_out = pl.n_out;
        L->spatial_out = pl.spatial_out;
        L->C = pl.C; L->H = pl.H; L->W = pl.W;
        net->layers.push_back(std::move(L));
    });
}

dpc_status dpc_network_add_skip(dpc_network* net, int32_t from_layer)
{
    return guarded([&] {
        DPC_REQUIRE(net, DPC_EINVAL, "dpc_network_add_skip: NULL network");
        DPC_REQUIRE(!net->finalized, DPC_ESTATE, "network already finalized");
        const int count = (int)net->layers.size();
        DPC_REQUIRE(count >= 1, DPC_EUNSUPPORTED, "dpc_network_add_skip: an Add layer cannot be the first layer");
        const Layer& below = *net->layers.back();
        DPC_REQUIRE(from_layer >= 0 && from_layer <= count - 1, DPC_EINVAL,
                    "dpc_network_add_skip: from_layer %d out of range [0, %d]", from_layer, count - 1);
        int sc = 0, sh = 0, sw = 0;
        const bool sp = net->spatial(from_layer, &sc, &sh, &sw);
        DPC_REQUIRE(net->size_of(from_layer) == below.n_out, DPC_EINVAL,
                    "dpc_network_add_skip: layer %d has %d neurons, the layer below the Add layer %d", from_layer,
                    net->size_of(from_layer), below.n_out);
        DPC_REQUIRE(sp == below.spatial_out && (!sp || (sc == below.C && sh == below.H && sw == below.W)), DPC_EINVAL,
                    "dpc_network_add_skip: the two operands differ in shape");
        auto L = std::make_unique<Layer>();
        L->kind = ADD;
        L->skip = from_layer;
        L->n_in = L->n_out = below.n_out;
        L->spatial_out = below.spatial_out;
        L->C = below.C; L->H = below.H; L->W = below.W;
        net->layers.push_back(std::move(L));
    });
}

dpc_status dpc_network_finalize(dpc_network* net, int32_t device)
{
    return guarded([&] {
        DPC_REQUIRE(net, DPC_EINVAL, "dpc_network_finalize: NULL network");
        DPC_REQUIRE(!net->finalized, DPC_ESTATE, "network already finalized");
        validate_chain(net);
        int ndev = 0;
        DPC_HIP(hipGetDeviceCount(&ndev));
        DPC_REQUIRE(device >= 0 && device < ndev, DPC_EINVAL, "device %d out of range (%d devices)", device, ndev);
        DeviceGuard guard(device);
        net->device = device;
        for (size_t i = 0; i < net->layers.size(); ++i) {
            Layer& L = *net->layers[i];
            if (L.kind == RELU) continue;
            if (L.kind == ADD) {
                // no weights; zero biases so that the ReLU step above it can fold "the bias of the layer below" as usual
                L.dBias.reserve(L.n_out);
                DPC_HIP(hipMemset(L.dBias.p, 0, (size_t)L.n_out * sizeof(float)));
                const int kb = net->layers[i - 1]->kind;
                L.unit_rows = kb != AFFINE && kb != CONV;
                if (L.spatial_out) {
                    // a 1x1 identity kernel: as the layer's own "cores" it is the Diagonal block of coefficient 1 on the operand
                    // below (used when that operand has no weight rows to start from), and it brings the zero channel biases
                    L.g = ConvGeom{L.C, L.H, L.W, L.C, 1, 1, 1, 0, L.H, L.W};
                    std::vector<float> eye((size_t)L.C * L.C, 0.0f), zb((size_t)L.C, 0.0f);
                    for (int c = 0; c < L.C; ++c) eye[(size_t)c * L.C + c] = 1.0f;
                    upload_conv_weights(L.g, eye.data(), zb.data(), L.cw);
                } else if (L.unit_rows) {
                    L.ldw = (int)round_up(L.n_out, kLdAlign);
                    std::vector<float> eye((size_t)round_up(L.n_out, 8) * L.ldw, 0.0f);
                    for (int r = 0; r < L.n_out; ++r) eye[(size_t)r * L.ldw + r] = 1.0f;
                    L.dW.reserve(eye.size());
                    DPC_HIP(hipMemcpy(L.dW.p, eye.data(), eye.size() * sizeof(float), hipMemcpyHostToDevice));
                }
                continue;
            }
            int pc, ph, pw;
            const bool prev_spatial = net->spatial((int)i, &pc, &ph, &pw);
            if (L.kind == AFFINE) {
                L.ldw = (int)round_up(L.n_in, kLdAlign);
                std::vector<float> w((size_t)round_up(L.n_out, 8) * L.ldw, 0.0f);   // rows padded to whole K groups of 8 (zeros)
                for (int r = 0; r < L.n_out; ++r)
                    for (int c = 0; c < L.n_in; ++c) {
                        int dst = c;                    // column c is a (C,H,W) index when the input is spatial
                        if (prev_spatial) {
                            const int x = c % pw, y = (c / pw) % ph, ch = c / (pw * ph);
                            dst = (y * pw + x) * pc + ch;
                        }
                        w[(size_t)r * L.ldw + dst] = L.hW[(size_t)r * L.n_in + c];
                    }
                L.dW.reserve(w.size());
                DPC_HIP(hipMemcpy(L.dW.p, w.data(), w.size() * sizeof(float), hipMemcpyHostToDevice));
                L.dBias.reserve(L.n_out);
                DPC_HIP(hipMemcpy(L.dBias.p, L.hb.data(), L.hb.size() * sizeof(float), hipMemcpyHostToDevice));
            } else {
                upload_conv_weights(L.g, L.hW.data(), L.hb.data(), L.cw);
                std::vector<float> bias((size_t)L.n_out);
                for (int i2 = 0; i2 < L.n_out; ++i2) bias[i2] = L.hb[i2 % L.g.Co];   // (H,W,C) order
                L.dBias.reserve(L.n_out);
                DPC_HIP(hipMemcpy(L.dBias.p, bias.data(), bias.size() * sizeof(float), hipMemcpyHostToDevice));
            }
        }
        // how many skip connections span one layer at most = how many blocks of rows can wait at once
        net->skip_depth = 0;
        for (size_t p = 0; p <= net->layers.size(); ++p) {
            int open = 0;
            for (size_t j = 0; j < net->layers.size(); ++j)
                if (net->layers[j]->kind == ADD && (size_t)net->layers[j]->skip <= p && p <= j) ++open;
            net->skip_depth = std::max(net->skip_depth, open);
        }
        // set-up for the certify calls: the pinned word the input validation reports into, and this device's address of
        // the library's static workspace
        DPC_HIP(hipHostMalloc(reinterpret_cast<void**>(&net->h_flag), sizeof(int32_t), hipHostMallocDefault));
        *net->h_flag = 0;
        (void)static_workspace(device);
        net->finalized = true;
    });
}

dpc_status dpc_network_destroy(dpc_network* net)
{
    return guarded([&] {
        if (!net) return;
        DPC_REQUIRE(net->live_results == 0, DPC_ESTATE, "destroy the network's results first");
        if (net->finalized) {
            DeviceGuard guard(net->device);
            delete net;
        } else {
            delete net;
        }
    });
}

dpc_status dpc_options_default(dpc_options* opt)
{
    return guarded([&] {
        DPC_REQUIRE(opt, DPC_EINVAL, "dpc_options_default: NULL");
        memset(opt, 0, sizeof *opt);
        opt->struct_size = (int32_t)sizeof(dpc_options);
        opt->max_backsub_depth = -1;
        opt->keep_symbolic = 0;
        opt->fuse = 1;
        opt->profile = 0;
        opt->use_graph = 1;
        opt->certifier = DPC_DEEPPOLY;
        opt->final_backsub_depth = DPC_SAME_DEPTH;
        opt->stream = nullptr;
    });
}

}  // extern "C"

namespace {

// Where the entry point that allocates nothing leaves its results (device pointers of the caller).
struct StaticOut {
    float* l; float* u; float* margin; int32_t* verdict;
};

// The certify call.  arena != NULL: the call of the entry point that allocates nothing -- the network's workspace has
// been swapped for one inside the arena, the result object lives there too and is dropped at the end, after its
// last-layer bounds, margins and verdicts have been copied to `so`.
void certify_impl(dpc_network* net, int32_t batch, const float* lo, const float* hi, const int32_t* label,
                  const dpc_options* opt_in, dpc_result** result, Arena* arena, const StaticOut* so)
{
    {
        DPC_REQUIRE(net && lo && hi && result, DPC_EINVAL, "dpc_certify: NULL argument");
        DPC_REQUIRE(net->finalized, DPC_ESTATE, "dpc_certify: network not finalized");
        const Tuning tuning = net->tuning();          // this network's knobs are the ones in force for the whole call
        TuningScope tuning_scope(&tuning);
        dpc_options opt;
        if (opt_in) {
            DPC_REQUIRE(opt_in->struct_size == (int32_t)sizeof(dpc_options), DPC_EINVAL,
                        "dpc_certify: options struct_size %d, expected %zu", opt_in->struct_size, sizeof(dpc_options));
            opt = *opt_in;
        } else {
            dpc_options_default(&opt);
        }
        DPC_REQUIRE(batch >= 0 && batch <= 16384, DPC_EINVAL, "dpc_certify: batch %d out of range [0, 16384]", batch);
        DPC_REQUIRE(opt.max_backsub_depth >= -1, DPC_EINVAL, "dpc_certify: max_backsub_depth must be >= -1");
        DPC_REQUIRE(opt.final_backsub_depth >= DPC_SAME_DEPTH, DPC_EINVAL, "dpc_certify: final_backsub_depth must be >= -2");
        if (opt.final_backsub_depth == DPC_SAME_DEPTH) opt.final_backsub_depth = opt.max_backsub_depth;
        DPC_REQUIRE(opt.keep_symbolic >= 0 && opt.keep_symbolic <= 2, DPC_EINVAL, "dpc_certify: keep_symbolic must be 0, 1 or 2");
        DPC_REQUIRE(opt.keep_symbolic == 0 || opt.final_backsub_depth == -1, DPC_EINVAL,
                    "dpc_certify: keep_symbolic needs a full traversal");
        DPC_REQUIRE(opt.keep_symbolic != 2 || opt.max_backsub_depth == -1, DPC_EINVAL,
                    "dpc_certify: keep_symbolic = 2 needs full traversals of every layer (max_backsub_depth = -1)");
        const int nl = (int)net->layers.size();
        const Layer& last = *net->layers[nl - 1];
        DPC_REQUIRE(opt.certifier == DPC_DEEPPOLY || opt.certifier == DPC_REUSECERT || opt.certifier == DPC_SKIPPOLY, DPC_EINVAL,
                    "dpc_certify: unknown certifier %d", opt.certifier);
        if (opt.certifier == DPC_SKIPPOLY) {
            // ReLU bounds over the neurons two layers back: a traversal replaces a ReLU layer and the layer under it in
            // one iteration, which is what the fused kernels execute; only the iteration count of a limit would differ
            DPC_REQUIRE(opt.max_backsub_depth == -1 && opt.final_backsub_depth == -1, DPC_EINVAL,
                        "dpc_certify: SkipPoly needs full traversals (max_backsub_depth = final_backsub_depth = -1)");
            DPC_REQUIRE(net->skip_depth == 0, DPC_EUNSUPPORTED, "dpc_certify: SkipPoly is specified for chain networks only");
        }
        const bool reuse_cert = opt.certifier == DPC_REUSECERT;
        if (arena) {
            DPC_REQUIRE(!reuse_cert && opt.keep_symbolic == 0 && contract_split_terms() == 0, DPC_EUNSUPPORTED,
                        "dpc_certify_static: DeepPoly (any depth limit) with keep_symbolic = 0 and the fp32 contraction only");
            opt.profile = 0;
            opt.use_graph = 0;
        }
        if (reuse_cert) {
            DPC_REQUIRE(opt.max_backsub_depth == -1 && opt.final_backsub_depth == -1 && opt.keep_symbolic == 0, DPC_EINVAL,
                        "dpc_certify: ReuseCert needs max_backsub_depth = -1 and keep_symbolic = 0");
            DPC_REQUIRE(nl % 2 == 1, DPC_EUNSUPPORTED, "dpc_certify: ReuseCert needs affine and ReLU layers alternating");
            for (int i = 0; i < nl; ++i) {
                const int kd = net->layers[i]->kind;
                DPC_REQUIRE(i % 2 ? kd == RELU : (kd == AFFINE || kd == CONV), DPC_EUNSUPPORTED,
                            "dpc_certify: ReuseCert covers chain networks with affine / convolution and ReLU layers alternating");
            }
        }
        if (net->skip_depth > 0)
            DPC_REQUIRE(!reuse_cert, DPC_EUNSUPPORTED, "dpc_certify: ReuseCert is specified for chain networks only");
        if (label) DPC_REQUIRE(last.kind == AFFINE && last.n_out >= 2, DPC_EUNSUPPORTED,
                               "dpc_certify: a label needs a fully-connected last layer with >= 2 outputs");
        DeviceGuard guard(net->device);
        hipStream_t s = reinterpret_cast<hipStream_t>(opt.stream);
        const int B = batch, n0 = net->n0, nK = last.n_out;

        // ---- result object (reused when compatible) ----
        dpc_result* res = *result;
        if (res) DPC_REQUIRE(res->net == net && res->batch == batch && res->keep_symbolic == opt.keep_symbolic,
                             DPC_EINVAL, "dpc_certify: the result passed in belongs to another network, batch or mode");
        std::unique_ptr<dpc_result> fresh;
        if (!res) {
            fresh.reset(arena ? new dpc_result(arena) : new dpc_result());
            res = fresh.get();
            res->net = net;
            res->batch = batch;
            res->keep_symbolic = opt.keep_symbolic;
            size_t tot = 0;
            for (int i = 0; i <= nl; ++i) {
                tot += 2 * (size_t)B * net->size_of(i);
                if (i > 0 && net->layers[i - 1]->kind == RELU) tot += 3 * (size_t)B * net->size_of(i);
            }
            res->pool.reserve(std::max<size_t>(tot, 1));
            res->l.assign(nl + 1, nullptr); res->u.assign(nl + 1, nullptr);
            res->lam.assign(nl + 1, nullptr); res->mu.assign(nl + 1, nullptr); res->nu.assign(nl + 1, nullptr);
            float* p = res->pool.p;
            for (int i = 0; i <= nl; ++i) {
                const size_t c = (size_t)B * net->size_of(i);
                res->l[i] = p; p += c;
                res->u[i] = p; p += c;
                if (i > 0 && net->layers[i - 1]->kind == RELU) {
                    res->lam[i] = p; p += c;
                    res->mu[i] = p; p += c;
                    res->nu[i] = p; p += c;
                }
            }
            res->margin.reserve(std::max<size_t>((size_t)B * (nK - 1), 1));
            res->verdict.reserve(std::max(B, 1));
            res->label.reserve(std::max(B, 1));
            res->sym_c.resize(nl + 2);
            res->sym_k.resize(nl + 2);
            res->sym_have.assign(nl + 2, 0);
            for (int i = 1; i <= nl + 1 && opt.keep_symbolic; ++i) {
                // 1: the last layer and the property's rows; 2: every affine / convolution / Add layer as well
                const bool kept = i >= nl || (opt.keep_symbolic == 2 && net->layers[i - 1]->kind != RELU);
                if (!kept) continue;
                const size_t rows = i <= nl ? 2 * (size_t)B * net->size_of(i) : (size_t)B * (nK - 1);
                res->sym_c[i].reset(new DevBuf<float>());
                res->sym_k[i].reset(new DevBuf<double>());
                res->sym_c[i]->reserve(std::max<size_t>(rows * net->ld_of(0), 1));
                res->sym_k[i]->reserve(std::max<size_t>(rows, 1));
            }
        }
        res->has_label = label != nullptr;
        res->certifier = opt.certifier;
        std::fill(res->sym_have.begin(), res->sym_have.end(), 0);
        memset(&res->prof, 0, sizeof res->prof);
        res->prof.struct_size = (int32_t)sizeof(dpc_profile);

        // ---- workspace ----
        size_t need_rows = 1;
        // rows per (side, input) group of the merged output + margin pass: padded up to the smallest group the fused
        // contraction epilogue takes, so that this pass can use it too
        const size_t RsMax = std::max<size_t>(2 * (size_t)nK - 1, 32);
        const size_t stage_need = std::max(2 * (size_t)B * n0, 2 * (size_t)B * RsMax) + 16;   // box staging / merged last pass + one flag word
        for (int i = 1; i <= nl; ++i)
            if (net->layers[i - 1]->kind != RELU) need_rows = std::max(need_rows, 2 * (size_t)B * net->size_of(i));
        need_rows = std::max(need_rows, 2 * (size_t)B * RsMax);   // output + margin rows of the last pass
        size_t need = workspace_floats(net, B, label != nullptr);
        const int ldE = (int)round_up(n0 + 1, kLdAlign);          // ReuseCert: input-level expression rows
        // ReuseCert on a convolutional front: the stored bounds of convolution layer i reach only its neurons' receptive
        // field, rwin[i] (ld == 0: rows over the whole input).  Kept while the window is smaller than the input.
        std::vector<ReuseWindow> rwin(nl + 2, ReuseWindow{0, 0, 0, 0, 0, 0});
        if (reuse_cert && tune(TK_REUSE_PATCH) && net->in_spatial) {
            ReuseWindow w{0, 0, net->inC, 1, 0, 0};
            w.ph = w.pw = 1;
            for (int i = 1; i <= nl && net->layers[i - 1]->kind == CONV; i += 2) {
                const ConvGeom& g = net->layers[i - 1]->g;
                ReuseWindow o{(g.kh - 1) * w.S + w.ph, (g.kw - 1) * w.S + w.pw, w.C0, g.stride * w.S, g.pad * w.S + w.P, 0};
                if ((size_t)o.ph * o.pw * o.C0 >= (size_t)n0) break;
                o.ld = (int)round_up((size_t)o.ph * o.pw * o.C0 + 1, kLdAlign);
                rwin[i] = o;
                w = o;
            }
        }
        // layers whose replacement step runs as an implicit contraction over the rows of the convolution layer two below
        auto implicit_step = [&](int k) {
            if (!reuse_cert || !tune(TK_REUSE_WINDOW) || k < 3 || k > nl || !net->in_spatial) return false;
            const Layer& Lk = *net->layers[k - 1];
            const Layer& Lb = *net->layers[k - 3];
            // the rows it reads: windows of the convolution layer two below, else rows over the image; 32-bit offsets inside
            // one input's block of rows and inside the workgroup index bound what the kernel takes
            const int64_t ld_in = rwin[k - 2].ld ? rwin[k - 2].ld : ldE;
            const int64_t positions = Lk.kind == CONV ? (int64_t)Lk.g.Ho * Lk.g.Wo : 1;
            const int64_t rows_m = Lk.kind == CONV ? Lk.g.Co : Lk.n_out;
            if ((2 * (int64_t)Lk.n_in + 1) * ld_in * 4 >= ((int64_t)1 << 31) || (int64_t)B * positions * rows_m >= ((int64_t)1 << 28)) return false;
            if (Lk.kind == CONV) return reuse_window_covers(Lk.g.Ci);
            return Lk.kind == AFFINE && Lb.kind == CONV && rwin[k - 2].ld != 0 && reuse_window_covers(Lb.g.Co) && !(k == nl && label);
        };
        if (reuse_cert) {
            size_t nmax = 1;
            for (int i = 1; i <= nl; i += 2) nmax = std::max<size_t>(nmax, net->size_of(i));
            const size_t Rm = 2 * (size_t)nK - 1;
            need = std::max(need, 2 * (size_t)B * std::max(nmax, Rm) * ldE);
            need = std::max(need, (size_t)B * (2 * nmax + 1) * ldE);
            if (label) need = std::max(need, 2 * (size_t)B * Rm * ((size_t)net->ld_of(nl - 1) + ldE));   // last step: rows + results
        }
        bool moved = net->ws->buf[0].reserve(need);
        moved |= net->ws->buf[1].reserve(need);
        if ((int)net->ws->skipbuf.size() < net->skip_depth) net->ws->skipbuf.resize(net->skip_depth);
        for (auto& sb : net->ws->skipbuf) {
            if (!sb) sb.reset(net->ws->fresh_buf());
            moved |= sb->reserve(need);
        }
        const bool fuse = opt.fuse && (opt.max_backsub_depth < 0 || opt.final_backsub_depth < 0);
        if (fuse) {
            size_t fuse_rows = 0;          // rows of the passes that can use fused epilogues (dense rows of FC layers)
            for (int i = 1; i <= nl; ++i)
                if (net->layers[i - 1]->kind == AFFINE) fuse_rows = std::max(fuse_rows, 2 * (size_t)B * net->size_of(i));
            if (label && last.kind == AFFINE) fuse_rows = std::max(fuse_rows, 2 * (size_t)B * RsMax);
            if (fuse_rows > 0 && fuse_rows * dpc_network::kMaxSlots * 4 <= ((size_t)1 << 31)) {
                moved |= net->ws->part.reserve(fuse_rows * dpc_network::kMaxSlots);
                net->ws->part_stride = std::max<int64_t>(net->ws->part_stride, (int64_t)fuse_rows);
            }
            if (nl >= 3 && net->layers[0]->kind == CONV && net->layers[0]->g.Ci <= 4 && net->layers[1]->kind == RELU)
                moved |= net->ws->pk2.reserve((size_t)B * net->ld_of(2) * 2);
            if ((int)net->ws->pk2v.size() != nl + 1) net->ws->pk2v.resize(nl + 1);
            size_t rrows = 0;
            for (int i = 3; i <= nl; ++i)
                if (net->layers[i - 1]->kind == RELU && net->layers[i - 2]->kind == CONV && net->layers[i - 2]->g.Ci > 4)
                    for (int k = i + 1; k <= nl; ++k)
                        if (net->layers[k - 1]->kind != RELU) rrows = std::max(rrows, 2 * (size_t)B * net->size_of(k));
            if (label) rrows = std::max(rrows, 2 * (size_t)B * RsMax);
            if (rrows > 0) moved |= net->ws->rpart.reserve(rrows);
            for (int i = 3; i <= nl; ++i) {
                if (net->layers[i - 1]->kind != RELU || net->layers[i - 2]->kind != CONV || net->layers[i - 2]->g.Ci <= 4) continue;
                if (!net->ws->pk2v[i]) net->ws->pk2v[i].reset(net->ws->fresh_buf());
                moved |= net->ws->pk2v[i]->reserve((size_t)B * net->ld_of(i) * 2);
            }
            if (net->ws->pk.size() != (size_t)nl + 1) net->ws->pk.resize(nl + 1);
            for (int i = 0; i <= nl; ++i) {
                const bool want = i == 0 ? !net->in_spatial || true : net->layers[i - 1]->kind == RELU;
                if (!want) continue;
                if (!net->ws->pk[i]) net->ws->pk[i].reset(net->ws->fresh_buf());
                moved |= net->ws->pk[i]->reserve((size_t)2 * B * net->ld_of(i) * 4);
            }
        }
        if (reuse_cert) {
            // split weights of every affine layer but the first (once), and room for the split rows of the last step
            size_t gather_need = 0;
            for (int i = 3; i <= nl; i += 2) {
                Layer& L = *net->layers[i - 1];
                if (L.kind == CONV && !implicit_step(i)) {
                    // a chunk of output positions at a time: at most 1 GiB of gathered rows, at least one position
                    const size_t per_pos = (size_t)(2 * L.g.kh * L.g.kw * L.g.Ci + 1) * (rwin[i].ld ? rwin[i].ld : ldE);
                    const size_t all = (size_t)B * L.g.Ho * L.g.Wo * per_pos;
                    gather_need = std::max(gather_need, std::min(all, std::max(per_pos, ((size_t)1 << 28) / per_pos * per_pos)));
                }
                if (L.dSplit[0].p) continue;
                if (L.kind == CONV) {
                    // the layer's weight matrix is its expanded kernel: [K+ | K- | b] over the (ky, kx, ci) window, per output channel
                    const int kk = L.g.kh * L.g.kw * L.g.Ci;
                    L.ld_split = (int)round_up(2 * kk + 1, kLdAlign);
                    for (int side = 0; side < 2; ++side) {
                        L.dSplit[side].reserve((size_t)L.g.Co * L.ld_split);
                        launch_reuse_split(L.cw.core, L.cw.ld_core, L.cw.bias_c, nullptr, L.g.Co, kk, L.dSplit[side].p, L.ld_split, 0, side, s);
                    }
                    continue;
                }
                L.ld_split = (int)round_up(2 * L.n_in + 1, kLdAlign);
                for (int side = 0; side < 2; ++side) {
                    L.dSplit[side].reserve((size_t)L.n_out * L.ld_split);
                    launch_reuse_split(L.dW.p, L.ldw, L.dBias.p, nullptr, L.n_out, L.n_in, L.dSplit[side].p, L.ld_split, 0, side, s);
                }
            }
            if (gather_need) moved |= net->ws->gather.reserve(gather_need);
            if (nl >= 3 && net->layers[0]->kind == CONV && !rwin[1].ld && !net->layers[0]->dDense.p) {
                // first layer: its neurons' expressions over the input are the expanded kernel rows, written out once
                Layer& L1 = *net->layers[0];
                const ConvGeom& g = L1.g;
                L1.dDense.reserve((size_t)L1.n_out * net->ld_of(0));
                moved |= net->ws->cst.reserve(L1.n_out);
                launch_fill_zero(L1.dDense.p, (int64_t)L1.n_out * net->ld_of(0), s);
                launch_expand_patch_rows(L1.cw.core, L1.cw.ld_core, g.Co, nullptr, L1.cw.bias_c, L1.n_out, L1.n_out, g.Co, g.Wo, g.kh, g.kw, g.Ci,
                                         g.stride, g.pad, g.H, g.W, L1.dDense.p, net->ld_of(0), net->ws->cst.p, s);
            }
            if (nl >= 3 && label) moved |= net->ws->rc_rows.reserve(2 * (size_t)B * (2 * (size_t)nK - 1) * net->layers[nl - 1]->ld_split);
        }
        if (const int terms = contract_split_terms()) {
            for (int i = 1; i <= nl; ++i) {
                Layer& L = *net->layers[i - 1];
                if (L.kind != AFFINE || L.n_out % 4 != 0 || L.wt_terms == terms) continue;
                int ldk, npad;
                L.dWt.release();
                L.dWt.reserve(split_weights_elems(L.n_out, L.n_in, terms, &ldk, &npad));
                launch_split_weights(L.dW.p, L.n_out, L.n_in, L.ldw, terms, L.dWt.p, s);
                L.wt_terms = terms;
            }
        }
        moved |= net->ws->cst.reserve(need_rows);
        moved |= net->ws->stage.reserve(stage_need);
        if (moved) ++net->ws->ws_epoch;

        if (B == 0) {
            if (fresh && !arena) { *result = fresh.release(); net->live_results++; }
            return;
        }

        Prof prof;
        prof.on = opt.profile != 0;
        prof.s = s;
        hipEvent_t t0 = nullptr, t1 = nullptr;
        if (prof.on) { t0 = prof.get(); t1 = prof.get(); DPC_HIP(hipEventRecord(t0, s)); }

        // ---- box and labels to the device, in the internal neuron order ----
        const size_t box = (size_t)B * n0;
        // pointers into this device's memory: one kernel copies, reorders and validates
        auto on_device = [&](const void* p) {
            hipPointerAttribute_t at{};
            if (hipPointerGetAttributes(&at, p) != hipSuccess) { (void)hipGetLastError(); return false; }
            return at.type == hipMemoryTypeDevice && at.device == net->device;
        };
        const bool resident = B > 0 && on_device(lo) && on_device(hi) && (!label || on_device(label));
        // the packed form of the box (for the fused concretisation epilogues) is written by the kernel that takes the box in
        const bool packed0 = resident && fuse && !(reuse_cert && (int)net->layers.size() >= 3) && !net->ws->pk.empty() && net->ws->pk[0] &&
                             net->ws->pk[0]->p;
        DPC_REQUIRE(resident || !arena, DPC_EINVAL, "dpc_certify_static: lo, hi and label must be device memory of the network's device");
        *net->h_flag = 0;
        if (resident) {
            if (!net->ws->dflag.p) {
                // a fill kernel, not a memset: the call may sit inside a caller's graph capture
                net->ws->dflag.reserve(1);
                zero_word_enqueue(net->ws->dflag.p, s);
            }
            ingest_enqueue(lo, hi, label, res->l[0], res->u[0], label ? res->label.p : nullptr, B, n0, net->in_spatial ? net->inC : 0,
                           net->inH, net->inW, nK, net->ws->dflag.p, net->h_flag, s, packed0 ? net->ws->pk[0]->p : nullptr, net->ld_of(0));
        } else if (net->in_spatial) {
            DPC_HIP(hipMemcpyAsync(net->ws->stage.p, lo, box * 4, hipMemcpyDefault, s));
            DPC_HIP(hipMemcpyAsync(net->ws->stage.p + box, hi, box * 4, hipMemcpyDefault, s));
            launch_chw_to_hwc(net->ws->stage.p, res->l[0], B, net->inC, net->inH, net->inW, s);
            launch_chw_to_hwc(net->ws->stage.p + box, res->u[0], B, net->inC, net->inH, net->inW, s);
        } else {
            DPC_HIP(hipMemcpyAsync(res->l[0], lo, box * 4, hipMemcpyDefault, s));
            DPC_HIP(hipMemcpyAsync(res->u[0], hi, box * 4, hipMemcpyDefault, s));
        }
        if (label && !resident) DPC_HIP(hipMemcpyAsync(res->label.p, label, (size_t)B * 4, hipMemcpyDefault, s));
        // validate lo <= hi, finite, labels in range on the device; the flag word is read after the stream has been
        // synchronised at the end of the call (no round trip in front of the kernels)
        if (!resident)
            check_inputs_enqueue(res->l[0], res->u[0], box, label ? res->label.p : nullptr, B, nK,
                             reinterpret_cast<int32_t*>(net->ws->stage.p + 2 * box), net->h_flag, s);

        // Launch-bound workloads (small networks: tens of short kernels) replay the whole kernel sequence as one
        // HIP graph: captured the first time a result object is reused, keyed on everything that shapes it.
        const bool graphable = opt.use_graph && s != nullptr && !prof.on && !opt.keep_symbolic && !fresh;
        const dpc_result::GraphKey gkey{(opt.max_backsub_depth + 2) * 65536 + opt.final_backsub_depth + 2, (opt.fuse != 0) | (opt.certifier << 1) | (packed0 ? 256 : 0), label != nullptr, g_tuning_epoch.load() + (net->tuning_epoch << 32), net->ws->ws_epoch};
        const bool merge_final = label && !opt.keep_symbolic && nl >= 2 && tune(TK_MERGE_FINAL);
        auto enqueue_reusecert = [&]() {
            Pass P{net, res, &opt, s, &prof, B, -1, false};
            float* E = net->ws->buf[0].p;            // stored bounds of the current affine layer: [side][b][n][ldE]
            float* Rr = net->ws->buf[1].p;           // [b][2n + 1][ldE]: the ReLU layer's input-level bounds + unit row
            double* cst = net->ws->cst.p;
            // constants travel in column n0 of the rows; the concretisation kernel takes them as fp64 per row
            auto concretise_rows = [&](const float* rows, int R, float* out_l, float* out_u) {
                const int64_t M = 2 * (int64_t)B * R;
                prof.begin(P_CONC);
                launch_reuse_const(rows, ldE, n0, M, cst, s);
                launch_concretise(rows, ldE, cst, 2, B, R, n0, res->l[0], res->u[0], out_l, out_u, nullptr, 0, nullptr, s);
                prof.end();
                res->prof.concretise_launches++;
                res->prof.concretise_bytes += (double)M * n0 * 4.0;
            };
            auto concretise_window_rows = [&](const float* rows, const ReuseWindow& w, const ConvGeom& g, float* out_l, float* out_u) {
                const int R = g.Co * g.Ho * g.Wo;
                const int64_t M = 2 * (int64_t)B * R;
                const int elems = w.ph * w.pw * w.C0;
                prof.begin(P_CONC);
                launch_reuse_const(rows, w.ld, elems, M, cst, s);
                launch_concretise_patch(rows, w.ld, cst, 2, B, R, PatchGeom{g.Wo, g.Co, w.ph, w.pw, w.C0, w.S, w.P, net->inH, net->inW}, res->l[0],
                                        res->u[0], out_l, out_u, nullptr, 0, nullptr, s);
                prof.end();
                res->prof.concretise_launches++;
                res->prof.concretise_bytes += (double)M * elems * 4.0;
            };
            {   // first layer: L = U = W x + b is already over the input
                Layer& L1 = *net->layers[0];
                run_pass(P, 0, 2, L1.n_out, &L1, res->l[1], res->u[1], -1);
            }
            for (int i = 2; i <= nl; ++i) {
                Layer& L = *net->layers[i - 1];
                if (L.kind == RELU) {
                    const Layer& A = *net->layers[i - 2];
                    prof.begin(P_OTHER);
                    launch_relax_params(res->l[i - 1], res->u[i - 1], res->lam[i], res->mu[i], res->nu[i], res->l[i], res->u[i],
                                        (int64_t)B * L.n_out, s);
                    prof.end();
                    res->prof.other_launches++;
                    prof.begin(P_RELAX);
                    const ReuseWindow& w = rwin[i - 1];
                    const bool next_window = w.ld && i < nl && (rwin[i + 1].ld || implicit_step(i + 1));
                    if (next_window) {
                        // rows stay over the receptive field (the layer above is a convolution that keeps a window)
                        const int elems = w.ph * w.pw * w.C0;
                        launch_reuse_scale(i == 2 ? nullptr : E, A.cw.core, A.cw.ld_core, A.cw.bias_c, res->lam[i], res->mu[i], res->nu[i], B, L.n_out,
                                           elems, w.ld, Rr, s, A.g.Co);
                        res->prof.relax_bytes += (double)B * (2.0 * L.n_out + 1) * w.ld * (i == 2 ? 4.0 : 8.0);
                    } else if (w.ld) {
                        // the layer above needs rows over the whole input: written out while they are scaled
                        launch_reuse_scale_expand(i == 2 ? nullptr : E, A.cw.core, A.cw.ld_core, A.cw.bias_c, A.g.Co, res->lam[i], res->mu[i],
                                                  res->nu[i], B, L.n_out, w, A.g.Wo, A.g.Co, net->inH, net->inW, n0, ldE, Rr, s);
                        res->prof.relax_bytes += (double)B * (2.0 * L.n_out + 1) * (ldE + w.ld) * 4.0;
                    } else {
                        launch_reuse_scale(i == 2 ? nullptr : E, A.kind == CONV ? A.dDense.p : A.dW.p, A.kind == CONV ? net->ld_of(0) : A.ldw,
                                           A.dBias.p, res->lam[i], res->mu[i], res->nu[i], B, L.n_out, n0, ldE, Rr, s);
                        res->prof.relax_bytes += (double)B * (2.0 * L.n_out + 1) * ldE * (i == 2 ? 4.0 : 8.0);
                    }
                    prof.end();
                    res->prof.relax_launches++;
                    continue;
                }
                if (L.kind == CONV) {
                    // the replacement step through the expanded kernel: per output position (input, ho, wo) the contraction
                    // [K+ | K- | b] (Co rows) x gathered rows of Rr, a chunk of positions per launch
                    const int Kp = 2 * L.g.kh * L.g.kw * L.g.Ci + 1;
                    const int64_t npos = (int64_t)B * L.g.Ho * L.g.Wo;
                    const ReuseWindow& wo = rwin[i];
                    const int ldR = wo.ld ? wo.ld : ldE;                                  // floats per stored row of this layer
                    const int ncol = wo.ld ? wo.ph * wo.pw * wo.C0 + 1 : n0 + 1;
                    if (implicit_step(i)) {
                        // rows of the ReLU layer below as they are (windows, or rows over the image), placed inside the frame of
                        // each output position while they are contracted
                        const ReuseWindow image{net->inH, net->inW, net->inC, 0, 0, ldE};
                        const ReuseWindow& wi = rwin[i - 2].ld ? rwin[i - 2] : image;
                        prof.begin(P_CONTRACT);
                        res->prof.contract_flop += launch_reuse_window(L.dSplit[0].p, L.dSplit[1].p, L.ld_split, L.g.Co, Rr, L.n_in, wi, L.g,
                                                                       wo.ld ? wo.ph : net->inH, wo.ld ? wo.pw : net->inW, ldR, wo.S, wo.P, !wo.ld, B,
                                                                       E, s);
                        prof.end();
                        res->prof.contract_launches++;
                        if (wo.ld) concretise_window_rows(E, wo, L.g, res->l[i], res->u[i]);
                        else concretise_rows(E, L.n_out, res->l[i], res->u[i]);
                        continue;
                    }
                    const int64_t chunk = std::min<int64_t>({npos, (int64_t)(net->ws->gather.count / ((size_t)Kp * ldR)), 65535});
                    DPC_REQUIRE(chunk >= 1, DPC_ENOMEM, "ReuseCert: gather workspace too small");
                    for (int64_t z0 = 0; z0 < npos; z0 += chunk) {
                        const int64_t nz = std::min(chunk, npos - z0);
                        prof.begin(P_RELAX);
                        if (wo.ld) launch_reuse_gather_patch(Rr, L.n_in, rwin[i - 2], wo, L.g, z0, nz, net->ws->gather.p, s);
                        else launch_reuse_gather(Rr, L.n_in, ldE, L.g, z0, nz, net->ws->gather.p, s);
                        prof.end();
                        res->prof.relax_launches++;
                        res->prof.relax_bytes += (double)nz * Kp * ldR * 8.0;
                        prof.begin(P_CONTRACT);
                        for (int side = 0; side < 2; ++side)
                            launch_contract_batched(L.dSplit[side].p, 0, L.g.Co, Kp, L.ld_split, net->ws->gather.p, (int64_t)Kp * ldR, ncol, ldR,
                                                    E + ((size_t)side * B * L.n_out + (size_t)z0 * L.g.Co) * ldR, (int64_t)L.g.Co * ldR, ldR,
                                                    (int)nz, s);
                        prof.end();
                        res->prof.contract_launches += 2;
                        res->prof.contract_flop += 2.0 * 2.0 * (double)nz * L.g.Co * Kp * ncol;
                    }
                    if (wo.ld) concretise_window_rows(E, wo, L.g, res->l[i], res->u[i]);
                    else concretise_rows(E, L.n_out, res->l[i], res->u[i]);
                    continue;
                }
                const int K = 2 * L.n_in + 1;
                const bool is_last = i == nl;
                if (implicit_step(i)) {
                    // first fully-connected layer above the convolutions: a convolution whose kernel covers the whole grid
                    const Layer& cv = *net->layers[i - 3];
                    const ConvGeom fc{cv.g.Co, cv.g.Ho, cv.g.Wo, L.n_out, cv.g.Ho, cv.g.Wo, 1, 0, 1, 1};
                    prof.begin(P_CONTRACT);
                    res->prof.contract_flop += launch_reuse_window(L.dSplit[0].p, L.dSplit[1].p, L.ld_split, L.n_out, Rr, L.n_in, rwin[i - 2], fc,
                                                                   net->inH, net->inW, ldE, 0, 0, true, B, E, s);
                    prof.end();
                    res->prof.contract_launches++;
                    concretise_rows(E, L.n_out, res->l[i], res->u[i]);
                    continue;
                }
                if (!is_last || !label) {
                    // stored bounds of the layer: [W+ | W- | b] Rr[b] (lower), [W- | W+ | b] Rr[b] (upper)
                    prof.begin(P_CONTRACT);
                    for (int side = 0; side < 2; ++side)
                        launch_contract_batched(L.dSplit[side].p, 0, L.n_out, K, L.ld_split, Rr, (int64_t)K * ldE, n0 + 1, ldE,
                                                E + (size_t)side * B * L.n_out * ldE, (int64_t)L.n_out * ldE, ldE, B, s);
                    prof.end();
                    res->prof.contract_launches += 2;
                    res->prof.contract_flop += 2.0 * 2.0 * B * (double)L.n_out * K * (n0 + 1);
                    concretise_rows(E, L.n_out, res->l[i], res->u[i]);
                } else {
                    // last layer with a property: output rows and margin rows (label-dependent, so per input) in one step
                    const int Rm = 2 * nK - 1;
                    const int64_t rows = 2 * (int64_t)B * Rm;
                    float* Fr = net->ws->buf[0].p;                                   // rows over the last hidden layer
                    float* T = net->ws->buf[0].p + (size_t)rows * net->ld_of(nl - 1); // their input-level expressions
                    prof.begin(P_OTHER);
                    launch_final_rows(L.dW.p, L.ldw, L.dBias.p, res->label.p, B, nK, L.n_in, Fr, net->ld_of(nl - 1), cst, s);
                    launch_reuse_split(Fr, net->ld_of(nl - 1), nullptr, cst, rows, L.n_in, net->ws->rc_rows.p, L.ld_split, (int64_t)B * Rm, 0, s);
                    prof.end();
                    res->prof.other_launches += 2;
                    prof.begin(P_CONTRACT);
                    for (int side = 0; side < 2; ++side)
                        launch_contract_batched(net->ws->rc_rows.p + (size_t)side * B * Rm * L.ld_split, (int64_t)Rm * L.ld_split, Rm, K,
                                                L.ld_split, Rr, (int64_t)K * ldE, n0 + 1, ldE,
                                                T + (size_t)side * B * Rm * ldE, (int64_t)Rm * ldE, ldE, B, s);
                    prof.end();
                    res->prof.contract_launches += 2;
                    res->prof.contract_flop += 2.0 * 2.0 * B * (double)Rm * K * (n0 + 1);
                    float* tl = net->ws->stage.p;
                    float* tu = net->ws->stage.p + (size_t)B * Rm;
                    concretise_rows(T, Rm, tl, tu);
                    prof.begin(P_OTHER);
                    launch_split_final(tl, tu, B, nK, res->l[nl], res->u[nl], res->margin.p, res->verdict.p, s);
                    prof.end();
                    res->prof.other_launches++;
                }
            }
        };
        auto enqueue_all = [&]() {
            if (reuse_cert && nl >= 3) { enqueue_reusecert(); return; }
            if (fuse && !packed0) launch_pack_bounds(res->l[0], res->u[0], B, n0, net->ld_of(0), net->ws->pk[0]->p, s);
            Pass P{net, res, &opt, s, &prof, B, opt.max_backsub_depth, fuse};
            bool relu_done = false;           // the pass below this ReLU layer has written its parameters already
            Pass::NextRelu next{};
            for (int i = 1; i <= nl; ++i) {
                Layer& L = *net->layers[i - 1];
                if (L.kind == RELU && relu_done) { relu_done = false; continue; }
                P.next = nullptr;
                P.rider_done = false;
                if (fuse && L.kind == AFFINE && i < nl && net->layers[i]->kind == RELU) {
                    float* pk2 = i + 1 == 2 ? net->ws->pk2.p
                                            : ((int)net->ws->pk2v.size() > i + 1 && net->ws->pk2v[i + 1]) ? net->ws->pk2v[i + 1]->p : nullptr;
                    next = Pass::NextRelu{res->lam[i + 1], res->mu[i + 1], res->nu[i + 1], res->l[i + 1], res->u[i + 1], L.dBias.p, L.n_out,
                                          net->ld_of(i + 1), net->ws->pk[i + 1]->p, pk2};
                    P.next = &next;
                }
                if (L.kind == RELU) {
                    prof.begin(P_OTHER);
                    if (fuse) {
                        // the layer's parameters and their packed forms (for the fused epilogues and the kernels that apply
                        // the ReLU step while they load rows) in one launch
                        float* pk2 = i == 2 ? net->ws->pk2.p
                                            : ((int)net->ws->pk2v.size() > i && net->ws->pk2v[i]) ? net->ws->pk2v[i]->p : nullptr;
                        launch_relax_params_pack(res->l[i - 1], res->u[i - 1], res->lam[i], res->mu[i], res->nu[i], res->l[i], res->u[i],
                                                 net->layers[i - 2]->dBias.p, B, L.n_out, net->ld_of(i), net->ws->pk[i]->p, pk2, s);
                    } else {
                        launch_relax_params(res->l[i - 1], res->u[i - 1], res->lam[i], res->mu[i], res->nu[i], res->l[i], res->u[i],
                                            (int64_t)B * L.n_out, s);
                    }
                    prof.end();
                    res->prof.other_launches++;
                    continue;
                }
                if (merge_final && i == nl) continue;       // bounded together with the margins below
                P.maxd = i == nl ? opt.final_backsub_depth : opt.max_backsub_depth;
                if (L.kind == ADD) {
                    if (P.maxd == 0) {
                        // no traverse iteration: simplify_* over prev0 + prev1 adds the stored bounds of the two operands
                        prof.begin(P_CONC);
                        launch_add_vectors(res->l[i - 1], res->l[L.skip], res->l[i], (int64_t)B * L.n_out, s);
                        launch_add_vectors(res->u[i - 1], res->u[L.skip], res->u[i], (int64_t)B * L.n_out, s);
                        prof.end();
                        res->prof.concretise_launches += 2;
                        continue;
                    }
                    if (L.unit_rows) {
                        // the operand below is a ReLU or another Add layer: the expressions start as coefficient 1 on its
                        // neurons (unit rows: two Diagonal blocks with the one on the skip operand) and no iteration is taken yet
                        run_pass(P, i - 1, 2, L.n_out, &L, res->l[i], res->u[i], res->sym_c[i] ? i : -1, 1.0, L.skip, 0);
                        continue;
                    }
                    // expressions of its neurons: the rows of the layer below (one traverse iteration already taken)
                    // + a unit block on the skip operand
                    Layer& below = *net->layers[i - 2];
                    run_pass(P, i - 2, 2, L.n_out, &below, res->l[i], res->u[i], res->sym_c[i] ? i : -1, 1.0, L.skip, 1);
                    continue;
                }
                run_pass(P, i - 1, 2, L.n_out, &L, res->l[i], res->u[i], res->sym_c[i] ? i : -1);
                relu_done = P.rider_done;
            }
            P.next = nullptr;
            P.rider_done = false;
            P.maxd = opt.final_backsub_depth;
            if (merge_final) {
                // Output-layer rows and margin rows walk the same layers: one pass of 2*nK-1 rows per (side, input)
                // instead of two passes (the margins' upper-side rows are computed and dropped).
                const int Rm = 2 * nK - 1;
                // groups padded with zero rows to the fused epilogue's minimum when that route is open
                const int Rs = (fuse && !opt.keep_symbolic && Rm < 32) ? 32 : Rm;
                float* tl = net->ws->stage.p;
                float* tu = net->ws->stage.p + (size_t)B * Rs;
                prof.begin(P_OTHER);
                launch_final_rows(last.dW.p, last.ldw, last.dBias.p, res->label.p, B, nK, last.n_in, net->ws->buf[0].p,
                                  net->ld_of(nl - 1), net->ws->cst.p, s, Rs);
                prof.end();
                res->prof.other_launches++;
                const Pass::FinalSplit fin{nK, Rs, res->l[nl], res->u[nl], res->margin.p, res->verdict.p};
                P.fin = &fin;
                run_pass(P, nl - 1, 2, Rs, nullptr, tl, tu, -1, (double)(2 * nK + nK - 1) / (2.0 * Rs));
                P.fin = nullptr;
                if (!P.rider_done) {
                    prof.begin(P_OTHER);
                    launch_split_final(tl, tu, B, nK, res->l[nl], res->u[nl], res->margin.p, res->verdict.p, s, Rs);
                    prof.end();
                    res->prof.other_launches++;
                }
            } else if (label) {
                const int nq = nK - 1;
                prof.begin(P_OTHER);
                launch_margin_rows(last.dW.p, last.ldw, last.dBias.p, res->label.p, B, nK, last.n_in, net->ws->buf[0].p,
                                   net->ld_of(nl - 1), net->ws->cst.p, s);
                prof.end();
                res->prof.other_launches++;
                run_pass(P, nl - 1, 1, nq, nullptr, res->margin.p, nullptr, res->sym_c[nl + 1] ? nl + 1 : -1);
                prof.begin(P_OTHER);
                launch_verdict(res->margin.p, B, nq, res->verdict.p, s);
                prof.end();
                res->prof.other_launches++;
            }
        };
        if (graphable && res->gexec && res->gkey == gkey) {
            res->prof = res->gprof;
            DPC_HIP(hipGraphLaunch(res->gexec, s));
        } else if (graphable) {
            if (res->gexec) { (void)hipGraphExecDestroy(res->gexec); res->gexec = nullptr; }
            DPC_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
            hipGraph_t graph = nullptr;
            try {
                enqueue_all();
            } catch (...) {
                (void)hipStreamEndCapture(s, &graph);
                if (graph) (void)hipGraphDestroy(graph);
                throw;
            }
            DPC_HIP(hipStreamEndCapture(s, &graph));
            hipGraphExec_t exec = nullptr;
            const hipError_t ie = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
            (void)hipGraphDestroy(graph);
            DPC_REQUIRE(ie == hipSuccess, DPC_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(ie));
            res->gexec = exec;
            res->gkey = gkey;
            res->gprof = res->prof;
            DPC_HIP(hipGraphLaunch(res->gexec, s));
        } else {
            enqueue_all();
        }
        prof.finish();
        if (prof.on) DPC_HIP(hipEventRecord(t1, s));
        if (so) {
            // results to the caller's device arrays, in the interface's neuron order
            const size_t cnt = (size_t)B * nK;
            if (last.spatial_out) {
                if (so->l) launch_hwc_to_chw(res->l[nl], so->l, B, last.C, last.H, last.W, s);
                if (so->u) launch_hwc_to_chw(res->u[nl], so->u, B, last.C, last.H, last.W, s);
            } else {
                if (so->l) DPC_HIP(hipMemcpyAsync(so->l, res->l[nl], cnt * sizeof(float), hipMemcpyDeviceToDevice, s));
                if (so->u) DPC_HIP(hipMemcpyAsync(so->u, res->u[nl], cnt * sizeof(float), hipMemcpyDeviceToDevice, s));
            }
            if (label && so->margin)
                DPC_HIP(hipMemcpyAsync(so->margin, res->margin.p, (size_t)B * (nK - 1) * sizeof(float), hipMemcpyDeviceToDevice, s));
            if (label && so->verdict)
                DPC_HIP(hipMemcpyAsync(so->verdict, res->verdict.p, (size_t)B * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
        }
        DPC_HIP(hipStreamSynchronize(s));
        {
            const int32_t h = *static_cast<volatile int32_t*>(net->h_flag);
            if (h && resident) zero_word_enqueue(net->ws->dflag.p, s);          // the next call expects a clean flag
            DPC_REQUIRE(!(h & 1), DPC_EINVAL, "dpc_certify: lo > hi or a non-finite bound");
            DPC_REQUIRE(!(h & 2), DPC_EINVAL, "dpc_certify: label out of range");
        }
        if (prof.on) {
            float ms = 0.f;
            DPC_HIP(hipEventElapsedTime(&ms, t0, t1));
            res->prof.total_ms = ms;
            for (auto& r : prof.segs) {
                DPC_HIP(hipEventElapsedTime(&ms, r.a, r.b));
                (r.cls == P_CONTRACT ? res->prof.contract_ms : r.cls == P_RELAX ? res->prof.relax_ms
                 : r.cls == P_CONC ? res->prof.concretise_ms : r.cls == P_CHAIN ? res->prof.chain_ms : res->prof.other_ms) += ms;
            }
        }
        if (fresh && !arena) { *result = fresh.release(); net->live_results++; }
    }
}

}  // namespace

extern "C" {

dpc_status dpc_certify(dpc_network* net, int32_t batch, const float* lo, const float* hi, const int32_t* label,
                       const dpc_options* opt, dpc_result** result)
{
    return guarded([&] { certify_impl(net, batch, lo, hi, label, opt, result, nullptr, nullptr); });
}

dpc_status dpc_certify_static(dpc_network* net, int32_t batch, const float* lo, const float* hi, const int32_t* label,
                              const dpc_options* opt, float* out_l, float* out_u, float* margin_lb, int32_t* verdict)
{
    return guarded([&] {
        DPC_REQUIRE(net && net->finalized, DPC_ESTATE, "dpc_certify_static: network not finalized");
        DPC_REQUIRE(label || (!margin_lb && !verdict), DPC_EINVAL, "dpc_certify_static: margins and verdicts need labels");
        DeviceGuard guard(net->device);
        Arena arena;
        arena.base = static_workspace(net->device);
        arena.size = kStaticWorkspaceBytes;
        // the call's workspace and result live in the static array; the network's own workspace is put back on every exit
        Workspace ws(&arena);
        struct Swap {
            dpc_network* n; Workspace* old;
            ~Swap() { n->ws = old; }
        } swap{net, net->ws};
        net->ws = &ws;
        dpc_result* none = nullptr;
        const StaticOut so{out_l, out_u, margin_lb, verdict};
        certify_impl(net, batch, lo, hi, label, opt, &none, &arena, &so);
    });
}


// ---- result accessors -------------------------------------------------------------------------

namespace {

// Copies a [batch, n] device array held in the internal neuron order to the caller, undoing the
// (H,W,C) storage of spatial layers.
void copy_out_layer(const dpc_result* res, int layer, const float* src, float* dst)
{
    if (!dst) return;
    const dpc_network* net = res->net;
    const size_t count = (size_t)res->batch * net->size_of(layer);
    if (count == 0) return;
    int C, H, W;
    if (net->spatial(layer, &C, &H, &W)) {
        DevBuf<float> tmp;
        tmp.reserve(count);
        launch_hwc_to_chw(src, tmp.p, res->batch, C, H, W, nullptr);
        DPC_HIP(hipMemcpy(dst, tmp.p, count * sizeof(float), hipMemcpyDefault));
    } else {
        DPC_HIP(hipMemcpy(dst, src, count * sizeof(float), hipMemcpyDefault));
    }
}

void require_result(const dpc_result* res, const char* who)
{
    DPC_REQUIRE(res && res->net, DPC_EINVAL, "%s: NULL result", who);
}

}  // namespace

dpc_status dpc_result_concrete(const dpc_result* res, int32_t layer, float* l, float* u)
{
    return guarded([&] {
        require_result(res, "dpc_result_concrete");
        DPC_REQUIRE(layer >= 0 && layer <= (int)res->net->layers.size(), DPC_EINVAL,
                    "dpc_result_concrete: layer %d out of range", layer);
        DeviceGuard guard(res->net->device);
        copy_out_layer(res, layer, res->l[layer], l);
        copy_out_layer(res, layer, res->u[layer], u);
    });
}

dpc_status dpc_result_relaxation(const dpc_result* res, int32_t relu_layer, float* lambda, float* mu, float* nu)
{
    return guarded([&] {
        require_result(res, "dpc_result_relaxation");
        DPC_REQUIRE(relu_layer >= 1 && relu_layer <= (int)res->net->layers.size() &&
                        res->net->layers[relu_layer - 1]->kind == RELU,
                    DPC_EINVAL, "dpc_result_relaxation: layer %d is not a ReLU layer", relu_layer);
        DeviceGuard guard(res->net->device);
        copy_out_layer(res, relu_layer, res->lam[relu_layer], lambda);
        copy_out_layer(res, relu_layer, res->mu[relu_layer], mu);
        copy_out_layer(res, relu_layer, res->nu[relu_layer], nu);
    });
}

namespace {

// Kept input-level expressions of `rows_per_input` rows per input (index `idx` of the result's store, side offset
// already applied by the caller through `side`) to the caller's arrays, in the interface's neuron orders.
void export_symbolic(const dpc_result* res, int idx, int side, int rows_per_input, bool rows_spatial, int rC, int rH, int rW,
                     float* coeff, float* cst)
{
    const dpc_network* net = res->net;
    const int B = res->batch, n0 = net->n0, ld0 = net->ld_of(0), n = rows_per_input;
    if (B == 0 || n == 0) return;
    int cC = 0, cH = 0, cW = 0;
    if (!net->spatial(0, &cC, &cH, &cW)) cC = 0;
    if (!rows_spatial) rC = 0;
    DevBuf<float> tmp, tmpk;
    if (coeff) tmp.reserve((size_t)n * n0);
    if (cst) tmpk.reserve(n);
    for (int b = 0; b < B; ++b) {
        const size_t row0 = ((size_t)side * B + b) * n;
        launch_sym_export(res->sym_c[idx]->p + row0 * ld0, ld0, res->sym_k[idx]->p + row0, n, n0, rC, rH, rW, cC, cH, cW,
                          coeff ? tmp.p : nullptr, cst ? tmpk.p : nullptr, nullptr);
        if (coeff) DPC_HIP(hipMemcpy(coeff + (size_t)b * n * n0, tmp.p, (size_t)n * n0 * sizeof(float), hipMemcpyDefault));
        if (cst) DPC_HIP(hipMemcpy(cst + (size_t)b * n, tmpk.p, (size_t)n * sizeof(float), hipMemcpyDefault));
    }
}

}  // namespace

dpc_status dpc_result_symbolic(const dpc_result* res, int32_t layer, int32_t side, float* coeff, float* cst)
{
    return guarded([&] {
        require_result(res, "dpc_result_symbolic");
        const Tuning tuning = res->net->tuning();
        TuningScope tuning_scope(&tuning);
        const dpc_network* net = res->net;
        const int nl = (int)net->layers.size();
        DPC_REQUIRE(layer >= 1 && layer <= nl, DPC_EINVAL, "dpc_result_symbolic: layer %d out of range [1, %d]", layer, nl);
        DPC_REQUIRE(net->layers[layer - 1]->kind != RELU, DPC_EINVAL,
                    "dpc_result_symbolic: layer %d is a ReLU layer (its polyhedral bounds are those of dpc_result_relaxation)", layer);
        DPC_REQUIRE(res->keep_symbolic >= 1 && res->sym_c[layer] && res->sym_have[layer], DPC_ESTATE,
                    "dpc_result_symbolic: the bounds of layer %d were not kept (keep_symbolic = 1 keeps the last layer, 2 every layer)", layer);
        DPC_REQUIRE(side == 0 || side == 1, DPC_EINVAL, "dpc_result_symbolic: side must be 0 or 1");
        DeviceGuard guard(net->device);
        int C = 0, H = 0, W = 0;
        const bool sp = net->spatial(layer, &C, &H, &W);
        export_symbolic(res, layer, side, net->size_of(layer), sp, C, H, W, coeff, cst);
    });
}

dpc_status dpc_result_relu_symbolic(const dpc_result* res, int32_t relu_layer, int32_t side, float* coeff, float* cst)
{
    return guarded([&] {
        require_result(res, "dpc_result_relu_symbolic");
        const Tuning tuning = res->net->tuning();
        TuningScope tuning_scope(&tuning);
        const dpc_network* net = res->net;
        const int nl = (int)net->layers.size();
        DPC_REQUIRE(relu_layer >= 2 && relu_layer <= nl && net->layers[relu_layer - 1]->kind == RELU, DPC_EINVAL,
                    "dpc_result_relu_symbolic: layer %d is not a ReLU layer", relu_layer);
        DPC_REQUIRE(res->certifier == DPC_SKIPPOLY, DPC_ESTATE, "dpc_result_relu_symbolic: certify was not run with certifier = DPC_SKIPPOLY");
        DPC_REQUIRE(side == 0 || side == 1, DPC_EINVAL, "dpc_result_relu_symbolic: side must be 0 or 1");
        const Layer& under = *net->layers[relu_layer - 2];
        DPC_REQUIRE(under.kind == AFFINE || under.kind == CONV, DPC_EUNSUPPORTED, "dpc_result_relu_symbolic: the layer under the ReLU layer has no weights");
        DeviceGuard guard(net->device);
        const int B = res->batch, n = under.n_out, below = relu_layer - 2, nb = net->size_of(below), ldb = net->ld_of(below);
        if (B == 0) return;
        int rC = 0, rH = 0, rW = 0, cC = 0, cH = 0, cW = 0;
        if (!net->spatial(relu_layer, &rC, &rH, &rW)) rC = 0;
        if (!net->spatial(below, &cC, &cH, &cW)) cC = 0;
        DevBuf<float> rows, out, outk;
        DevBuf<double> k;
        rows.reserve((size_t)n * ldb);
        k.reserve(n);
        if (coeff) out.reserve((size_t)n * nb);
        if (cst) outk.reserve(n);
        for (int b = 0; b < B; ++b) {
            // the rows of the layer under the ReLU layer (its own L = U), then scaled by lambda (L) or mu (U), nu added to U
            if (under.kind == AFFINE) {
                DPC_HIP(hipMemcpy2DAsync(rows.p, (size_t)ldb * 4, under.dW.p, (size_t)under.ldw * 4, (size_t)ldb * 4, n, hipMemcpyDeviceToDevice, nullptr));
            } else {
                const ConvGeom& g = under.g;
                launch_fill_zero(rows.p, (int64_t)n * ldb, nullptr);
                launch_expand_patch_rows(under.cw.core, under.cw.ld_core, g.Co, nullptr, under.cw.bias_c, n, n, g.Co, g.Wo, g.kh, g.kw, g.Ci,
                                         g.stride, g.pad, g.H, g.W, rows.p, ldb, k.p, nullptr);
            }
            const float* sc = (side == 0 ? res->lam[relu_layer] : res->mu[relu_layer]) + (size_t)b * n;
            launch_scale_rows(rows.p, ldb, n, nb, k.p, under.kind == AFFINE ? under.dBias.p : nullptr, sc,
                              side == 1 ? res->nu[relu_layer] + (size_t)b * n : nullptr, nullptr);
            launch_sym_export(rows.p, ldb, k.p, n, nb, rC, rH, rW, cC, cH, cW, coeff ? out.p : nullptr, cst ? outk.p : nullptr, nullptr);
            if (coeff) DPC_HIP(hipMemcpy(coeff + (size_t)b * n * nb, out.p, (size_t)n * nb * sizeof(float), hipMemcpyDefault));
            if (cst) DPC_HIP(hipMemcpy(cst + (size_t)b * n, outk.p, (size_t)n * sizeof(float), hipMemcpyDefault));
        }
    });
}

dpc_status dpc_result_margin_symbolic(const dpc_result* res, float* coeff, float* cst)
{
    return guarded([&] {
        require_result(res, "dpc_result_margin_symbolic");
        const Tuning tuning = res->net->tuning();
        TuningScope tuning_scope(&tuning);
        const dpc_network* net = res->net;
        const int nl = (int)net->layers.size();
        DPC_REQUIRE(res->keep_symbolic >= 1 && res->has_label && res->sym_c[nl + 1] && res->sym_have[nl + 1], DPC_ESTATE,
                    "dpc_result_margin_symbolic: certify was not run with keep_symbolic >= 1 and labels");
        DeviceGuard guard(net->device);
        export_symbolic(res, nl + 1, 0, net->size_of(nl) - 1, false, 0, 0, 0, coeff, cst);
    });
}

dpc_status dpc_result_verdict(const dpc_result* res, int32_t* verdict, float* margin_lb)
{
    return guarded([&] {
        require_result(res, "dpc_result_verdict");
        DPC_REQUIRE(res->has_label, DPC_ESTATE, "dpc_result_verdict: certify was run without labels");
        DeviceGuard guard(res->net->device);
        const int B = res->batch, nq = res->net->size_of((int)res->net->layers.size()) - 1;
        if (B == 0) return;
        if (verdict) DPC_HIP(hipMemcpy(verdict, res->verdict.p, (size_t)B * sizeof(int32_t), hipMemcpyDefault));
        if (margin_lb) DPC_HIP(hipMemcpy(margin_lb, res->margin.p, (size_t)B * nq * sizeof(float), hipMemcpyDefault));
    });
}

dpc_status dpc_result_profile(const dpc_result* res, dpc_profile* out)
{
    return guarded([&] {
        require_result(res, "dpc_result_profile");
        DPC_REQUIRE(out && out->struct_size == (int32_t)sizeof(dpc_profile), DPC_EINVAL,
                    "dpc_result_profile: out is NULL or its struct_size is not %zu", sizeof(dpc_profile));
        *out = res->prof;
        out->struct_size = (int32_t)sizeof(dpc_profile);
    });
}

dpc_status dpc_result_destroy(dpc_result* res)
{
    return guarded([&] {
        if (!res) return;
        DeviceGuard guard(res->net->device);
        res->net->live_results--;
        delete res;
    });
}

// ---- the hot kernels on caller-owned device buffers --------------------------------------------

dpc_status dpc_op_contract(const float* A, int64_t M, int32_t K, int32_t lda, const float* W, int32_t N, int32_t ldw,
                           float* Cout, int32_t ldc, void* stream)
{
    return guarded([&] { launch_contract(A, M, K, lda, W, N, ldw, Cout, ldc, reinterpret_cast<hipStream_t>(stream)); });
}

dpc_status dpc_op_relax_step(float* C, int32_t ldc, double* cst, int32_t nsides, int32_t batch, int32_t R, int32_t n,
                             const float* lambda, const float* mu, const float* nu, const float* bias,
                             const float* shared_src, int32_t ld_src, void* stream)
{
    return guarded([&] {
        launch_relax_step(C, ldc, cst, nsides, batch, R, n, lambda, mu, nu, bias, shared_src, ld_src, nullptr,
                          reinterpret_cast<hipStream_t>(stream));
    });
}

dpc_status dpc_op_concretise(const float* C, int32_t ldc, const double* cst, int32_t nsides, int32_t batch, int32_t R,
                             int32_t n, const float* lo, const float* hi, float* out_l, float* out_u, void* stream)
{
    return guarded([&] {
        launch_concretise(C, ldc, cst, nsides, batch, R, n, lo, hi, out_l, out_u, nullptr, 0, nullptr,
                          reinterpret_cast<hipStream_t>(stream));
    });
}

dpc_status dpc_op_conv_transpose(const float* in, int64_t M, int32_t ld_in, int32_t ih, int32_t iw, int32_t Co, int32_t Ci,
                                 int32_t kh, int32_t kw, int32_t stride, int32_t off, const float* K_host,
                                 float* out, int32_t ld_out, int32_t oh, int32_t ow, void* stream)
{
    return guarded([&] {
        DPC_REQUIRE(in && out && K_host && M >= 0, DPC_EINVAL, "dpc_op_conv_transpose: NULL argument");
        DPC_REQUIRE(ih >= 1 && iw >= 1 && Co >= 1 && Ci >= 1 && kh >= 1 && kw >= 1 && stride >= 1 && off >= 0 && oh >= 1 && ow >= 1,
                    DPC_EINVAL, "dpc_op_conv_transpose: bad geometry");
        DPC_REQUIRE(oh + off <= (ih - 1) * stride + kh && ow + off <= (iw - 1) * stride + kw, DPC_EINVAL,
                    "dpc_op_conv_transpose: output window exceeds the transposed convolution's extent");
        DPC_REQUIRE((int64_t)ih * iw * Co <= (1 << 24) && (int64_t)oh * ow * Ci <= (1 << 24), DPC_EINVAL,
                    "dpc_op_conv_transpose: rows too long");
        ConvGeom g{Ci, oh, ow, Co, kh, kw, stride, off, ih, iw};
        ConvWeights w;
        std::vector<float> zero_bias((size_t)Co, 0.0f);
        upload_conv_weights(g, K_host, zero_bias.data(), w);
        hipStream_t st = reinterpret_cast<hipStream_t>(stream);
        launch_conv_transpose_rows(in, M, ld_in, ih, iw, g, w, out, ld_out, oh, ow, off, st);
        DPC_HIP(hipStreamSynchronize(st));      // the temporary weights are freed on return
    });
}

dpc_status dpc_tuning_set(const char* key, int32_t value)
{
    return guarded([&] {
        DPC_REQUIRE(key, DPC_EINVAL, "dpc_tuning_set: NULL key");
        const int k = tune_key(key);
        DPC_REQUIRE(k >= 0, DPC_EINVAL, "dpc_tuning_set: unknown key '%s'", key);
        DPC_REQUIRE(k != TK_CONTRACT_SPLIT || value == 0 || value == 2 || value == 3, DPC_EINVAL,
                    "dpc_tuning_set: contract_split takes 0, 2 or 3");
        g_tune.v[k].store(value, std::memory_order_relaxed);
        ++g_tuning_epoch;
    });
}

dpc_status dpc_network_tuning_set(dpc_network* net, const char* key, int32_t value)
{
    return guarded([&] {
        DPC_REQUIRE(net && key, DPC_EINVAL, "dpc_network_tuning_set: NULL argument");
        const int k = tune_key(key);
        DPC_REQUIRE(k >= 0, DPC_EINVAL, "dpc_network_tuning_set: unknown key '%s'", key);
        DPC_REQUIRE(k != TK_CONTRACT_SPLIT || value == kTuneUnset || value == 0 || value == 2 || value == 3, DPC_EINVAL,
                    "dpc_network_tuning_set: contract_split takes 0, 2 or 3");
        net->tune_override[k] = value;
        ++net->tuning_epoch;
    });
}

}  // extern "C"
