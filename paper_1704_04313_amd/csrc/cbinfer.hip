// C ABI, network plan, per-layer state and the per-frame schedule.
// Every step of the path runs in the kernels declared in kernels.h; this file validates the
// network description, lays out device memory, uploads the filter matrices and enqueues the
// kernels of a frame on the caller's stream without ever waiting for the device.
#include "../../include/cbinfer.h"
#include "kernels.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

namespace {

thread_local std::string g_err = "";

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

constexpr size_t kAlign = 256;
constexpr int kMaxGemmGrid = 256; // workgroups of one GEMM launch (one per compute unit of an MI355X)
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline int words_for(long long bits) { return (int)((bits + 63) / 64); }

struct Op {
    int kind = 0;
    // input map
    int C = 0, Cs = 0, H = 0, W = 0;
    int pix_words = 0;   // CONV: 4-byte words per pixel of the input map (see GemmArgs::pix_words)
    // output map
    int M = 0, Ms = 0, Ho = 0, Wo = 0;
    int kh = 1, kw = 1, stride = 1, pad = 0, relu = 0, dense = 0, propagate = 0;
    float tau = 0.f;
    int K = 0, Kpad = 0, Mpad = 0;
    int gemm_grid = 0;
    bool select = false; // CONV: maps small enough for the GEMM (and the pooling after it) to pick their
                         // positions from the update maps themselves; index lists are then only
                         // extracted when the caller asks for them
    int pool_after = -1; // CONV: index of the pooling op that directly follows, or -1
    int conv_before = -1; // MAXPOOL: index of the conv it follows
    // workspace offsets (bytes); SIZE_MAX = absent
    size_t o_ref = SIZE_MAX, o_cur = SIZE_MAX, o_out = SIZE_MAX, o_wt = SIZE_MAX, o_bias = SIZE_MAX,
           o_taps = SIZE_MAX, o_chg = SIZE_MAX, o_upd = SIZE_MAX, o_pool = SIZE_MAX, o_clist = SIZE_MAX,
           o_ulist = SIZE_MAX, o_counts = SIZE_MAX, o_groups = SIZE_MAX;
};

struct Plan {
    std::vector<Op> ops;
    int S = 1, in_c = 0, in_h = 0, in_w = 0;
    bool hold = false;
    int dtype = cbk::kF32; // storage of maps and filter matrices
    size_t o_iota = 0, o_const = 0, o_partial = 0, o_tickets = 0;
    bool pipeline = false;     // two sets of per-frame scratch, so that consecutive frames may overlap
    size_t o_set0 = 0;         // first byte of the per-frame scratch (everything a frame writes except the stored maps)
    size_t set_bytes = 0;      // its size; with `pipeline` a second set follows directly behind it
    size_t o_flags = 0;        // the byte change maps of all layers behind the first, contiguous
    long long flag_words = 0;  // their total size in 64-bit words
    int compute_units = 256; // sizes the GEMM grids; the device's count replaces it in cbinfer_create
    int iota_len = 0;
    size_t bytes = 0;
};

struct Carver {
    size_t off = 0;
    size_t take(size_t bytes)
    {
        const size_t o = off;
        off += align_up(bytes ? bytes : 1);
        return o;
    }
};

// Validates the description and lays out the workspace.  Touches no device.
int make_plan(const cbinfer_network *net, float threshold, bool need_threshold, Plan &P)
{
    if (!net) return fail(CBINFER_EINVAL, "network description is NULL");
    if (net->n_layers <= 0 || !net->layers) return fail(CBINFER_EINVAL, "network has no layers");
    if (net->in_c <= 0 || net->in_h <= 0 || net->in_w <= 0)
        return fail(CBINFER_EINVAL, "frame shape must be positive (got %d x %d x %d)", net->in_c, net->in_h,
                    net->in_w);
    if (net->n_streams <= 0) return fail(CBINFER_EINVAL, "n_streams must be >= 1");
    if (net->dtype != CBINFER_F32 && net->dtype != CBINFER_BF16)
        return fail(CBINFER_EINVAL, "dtype must be CBINFER_F32 or CBINFER_BF16");
    if (net->flags & ~(uint32_t)(CBINFER_FLAG_HOLD_REFERENCE | CBINFER_FLAG_LISTS_EVERY_FRAME | CBINFER_FLAG_PIPELINE_FRAMES))
        return fail(CBINFER_EINVAL, "unknown flag bits");
    if (need_threshold && !(threshold >= 0.0f && std::isfinite(threshold))) {
        bool all_own = true;
        for (int l = 0; l < net->n_layers; ++l)
            if (net->layers[l].kind == CBINFER_OP_CONV && !(net->layers[l].threshold >= 0.0f)) all_own = false;
        if (!all_own) return fail(CBINFER_EINVAL, "global threshold must be finite and >= 0");
    }
    P.S = net->n_streams;
    P.in_c = net->in_c;
    P.in_h = net->in_h;
    P.in_w = net->in_w;
    P.hold = (net->flags & CBINFER_FLAG_HOLD_REFERENCE) != 0;
    // Frames in flight pay with event traffic between the two streams; a network of one or two
    // operations has nothing to overlap that would be worth it and runs on the caller's stream.
    P.pipeline = (net->flags & CBINFER_FLAG_PIPELINE_FRAMES) != 0 && net->n_layers >= 3;
    P.dtype = net->dtype == CBINFER_BF16 ? cbk::kBF16 : cbk::kF32;
    const int eu = cbk::elems_per_unit(P.dtype);
    const size_t esz = (size_t)cbk::elem_bytes(P.dtype);
    P.ops.clear();
    int c = net->in_c, h = net->in_h, w = net->in_w;
    const long long lim = (1ll << 31) - 1;
    long long max_px = 0;
    for (int l = 0; l < net->n_layers; ++l) {
        const cbinfer_layer &L = net->layers[l];
        Op op;
        op.kind = L.kind;
        op.C = c;
        op.Cs = round_up(c, eu);
        op.H = h;
        op.W = w;
        if (L.kind == CBINFER_OP_CONV) {
            if (L.cin != c) return fail(CBINFER_EINVAL, "layer %d: cin %d does not match incoming %d channels", l, L.cin, c);
            if (L.cout <= 0) return fail(CBINFER_EINVAL, "layer %d: cout must be positive", l);
            if (L.kh <= 0 || L.kw <= 0 || L.stride <= 0) return fail(CBINFER_EINVAL, "layer %d: kernel size and stride must be positive", l);
            if (L.pad < 0 || L.pad >= L.kh || L.pad >= L.kw) return fail(CBINFER_EINVAL, "layer %d: need 0 <= pad < kernel size", l);
            if (L.kh > 64 || L.kw > 64) return fail(CBINFER_EUNSUPPORTED, "layer %d: kernels larger than 64 are not supported", l);
            if (h + 2 * L.pad < L.kh || w + 2 * L.pad < L.kw) return fail(CBINFER_EINVAL, "layer %d: kernel larger than padded input", l);
            if (!L.weight) return fail(CBINFER_EINVAL, "layer %d: weight pointer is NULL", l);
            if (std::isnan(L.threshold) || std::isinf(L.threshold)) return fail(CBINFER_EINVAL, "layer %d: threshold must be finite", l);
            op.kh = L.kh;
            op.kw = L.kw;
            op.stride = L.stride;
            op.pad = L.pad;
            op.relu = L.relu != 0;
            op.dense = L.dense != 0;
            op.propagate = L.propagate != 0;
            if (op.propagate && l == 0) return fail(CBINFER_EINVAL, "layer 0: the first layer has no op before it to propagate changes from");
            if (op.propagate && op.dense) return fail(CBINFER_EINVAL, "layer %d: propagate and dense exclude each other", l);
            op.tau = L.threshold >= 0.0f ? L.threshold : threshold;
            op.M = L.cout;
            op.Ms = round_up(op.M, eu);
            op.Ho = (h + 2 * L.pad - L.kh) / L.stride + 1;
            op.Wo = (w + 2 * L.pad - L.kw) / L.stride + 1;
            op.K = L.kh * L.kw * op.Cs;
            op.Kpad = round_up(op.K, cbk::gemm_k_multiple(P.dtype));
            // A large camera frame of a float32 network with 1, 2, 3, 5, 6 or 7 channels is stored without
            // padding channels: the detection pass then moves only what the method needs.
            op.pix_words = (l == 0 && cbk::detect_frame_packs(P.dtype, op.C, (long long)P.S * h * w)) ? op.C
                                                                                                     : op.Cs * (int)esz / 4;
            if ((long long)P.S * h * w * op.pix_words + 4 > 0x7fffffffll)
                return fail(CBINFER_EUNSUPPORTED, "layer %d: input map beyond 2^31-1 4-byte words", l);
            op.Mpad = round_up(op.M, cbk::gemm_channel_tile(op.M));
            if (op.Kpad / cbk::gemm_k_multiple(P.dtype) >= (1 << 20))
                return fail(CBINFER_EUNSUPPORTED, "layer %d: more than 2^20 slices of 128 bytes per filter-matrix row", l);
            c = op.M;
        } else if (L.kind == CBINFER_OP_MAXPOOL) {
            if (L.kh != L.kw || L.kh < 1) return fail(CBINFER_EINVAL, "layer %d: pooling window must be square", l);
            if (L.stride != L.kh || L.pad != 0) return fail(CBINFER_EUNSUPPORTED, "layer %d: pooling needs stride == window and no padding", l);
            if (l == 0 || P.ops.back().kind != CBINFER_OP_CONV)
                return fail(CBINFER_EUNSUPPORTED, "layer %d: pooling must directly follow a convolution layer", l);
            if (h % L.kh || w % L.kh) return fail(CBINFER_EINVAL, "layer %d: map %d x %d is not a multiple of the pooling window", l, h, w);
            op.kh = op.kw = op.stride = L.kh;
            op.M = c;
            op.Ms = round_up(c, eu);
            op.Ho = h / L.kh;
            op.Wo = w / L.kh;
            op.conv_before = l - 1;
            P.ops.back().pool_after = l;
        } else {
            return fail(CBINFER_EINVAL, "layer %d: unknown kind %d", l, L.kind);
        }
        h = op.Ho;
        w = op.Wo;
        const long long in_elems = (long long)P.S * op.H * op.W * op.Cs;
        const long long out_elems = (long long)P.S * op.Ho * op.Wo * (L.kind == CBINFER_OP_CONV ? op.Ms : op.Ms);
        if (in_elems > lim || out_elems > lim || (long long)op.Mpad * op.Kpad > lim)
            return fail(CBINFER_EUNSUPPORTED, "layer %d: a map or the filter matrix exceeds 2^31-1 elements", l);
        max_px = std::max(max_px, std::max((long long)P.S * op.H * op.W, (long long)P.S * op.Ho * op.Wo));
        P.ops.push_back(op);
    }
    // workspace layout: what persists from frame to frame first ...
    Carver cv;
    for (size_t l = 0; l < P.ops.size(); ++l) {
        Op &op = P.ops[l];
        const size_t in_px = (size_t)P.S * op.H * op.W, out_px = (size_t)P.S * op.Ho * op.Wo;
        // every map is followed by one 16-byte unit of zeros, which gathers outside the image read
        op.o_out = cv.take(out_px * op.Ms * esz + 16);
        if (op.kind == CBINFER_OP_CONV) {
            // Layers behind the first keep no copy of their previous input unless asked to hold it
            // or to run densely: their previous input is the stored output of the op before them.
            if (l == 0 || ((P.hold || op.dense) && !op.propagate)) op.o_ref = cv.take(in_px * op.pix_words * 4 + 16);
            if (l == 0 && P.hold) op.o_cur = cv.take(in_px * op.pix_words * 4 + 16);
            op.o_wt = cv.take((size_t)op.Mpad * op.Kpad * esz);
            op.o_bias = cv.take((size_t)op.Mpad * 4);
            op.o_taps = cv.take((size_t)op.Kpad / eu * sizeof(int2));
        }
    }
    P.iota_len = (int)max_px;
    P.o_iota = cv.take((size_t)P.iota_len * 4);
    P.o_const = cv.take(P.ops.size() * 2 * 4);
    // ... then everything a frame writes besides the stored maps: change maps, index lists, counters,
    // the multiplication kernel's partial sums and tickets.  Two such sets when consecutive frames
    // may overlap; state->at() picks the set of the frame in hand.
    P.o_set0 = cv.off;
    for (size_t l = 0; l < P.ops.size(); ++l) {
        Op &op = P.ops[l];
        const size_t in_px = (size_t)P.S * op.H * op.W, out_px = (size_t)P.S * op.Ho * op.Wo;
        op.o_ulist = cv.take(out_px * 4);
        op.o_counts = cv.take(4 * 4);
        if (op.kind == CBINFER_OP_CONV) {
            // change map of the first layer: one bit per pixel
            if (l == 0) op.o_chg = cv.take(((size_t)words_for((long long)in_px) + 1) * 8);
            op.o_upd = cv.take(((size_t)words_for((long long)out_px) + 1) * 8);
            if (op.pool_after >= 0) {
                const Op &pp = P.ops[op.pool_after];
                op.o_pool = cv.take(((size_t)words_for((long long)P.S * pp.Ho * pp.Wo) + 1) * 8);
            }
            op.o_clist = cv.take(in_px * 4);
            // group counts of the three maps condensed per layer (changed, update, pooled)
            op.o_groups = cv.take(3 * cbk::compact_group_count_bytes(words_for((long long)std::max(in_px, out_px))));
        }
    }
    // Change maps of the layers behind the first: one bit per pixel, or one byte per pixel when the
    // op before fills it in.  Contiguous, so that one range clear at the start of a frame covers them.
    P.o_flags = cv.off;
    for (size_t l = 1; l < P.ops.size(); ++l) {
        Op &op = P.ops[l];
        if (op.kind != CBINFER_OP_CONV) continue;
        op.o_chg = cv.take(((size_t)words_for((long long)P.S * op.H * op.W) + 1) * 64);
    }
    P.flag_words = (long long)(cv.off - P.o_flags) / 8;
    for (Op &op : P.ops)
        if (op.kind == CBINFER_OP_CONV)
            op.select = !(net->flags & CBINFER_FLAG_LISTS_EVERY_FRAME) &&
                        words_for((long long)P.S * op.Ho * op.Wo) <= cbk::gemm_select_max_words() &&
                        words_for((long long)P.S * op.H * op.W) <= cbk::gemm_select_max_words();
    {
        // sized for the largest grid the GEMM may use (its cap), whatever the device turns out to be
        size_t pb = 0;
        for (const Op &op : P.ops)
            if (op.kind == CBINFER_OP_CONV) pb = std::max(pb, cbk::gemm_partial_bytes(op.M, kMaxGemmGrid));
        P.o_partial = cv.take(pb);
        P.o_tickets = cv.take(cbk::gemm_ticket_bytes(kMaxGemmGrid));
    }
    P.set_bytes = cv.off - P.o_set0;
    if (P.pipeline) cv.off += P.set_bytes;
    P.bytes = cv.off;
    return CBINFER_OK;
}

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    int layer = 0, step = 0;
};

} // namespace

struct cbinfer_state {
    Plan plan;
    hipStream_t stream = nullptr;
    char *ws = nullptr;
    bool owns_ws = false;
    // Frames in flight (CBINFER_FLAG_PIPELINE_FRAMES): consecutive frames alternate between two
    // streams of the library's own and between the two scratch sets; events order every kernel that
    // overwrites a stored map behind the previous frame's readers of that map.
    hipStream_t pstream[2] = {nullptr, nullptr};
    hipEvent_t ev_in = nullptr;
    std::vector<hipEvent_t> ev_op[2]; // per slot: one per operation (its last kernel) and one for the output copy
    hipStream_t work = nullptr;       // the stream the kernels of the frame in hand (and of later queries) go to
    int par = 0;                      // scratch set of the frame in hand / of the last frame
    bool have_prev = false;           // a frame is (possibly still) running on the other stream
    int pipe_gap = 3;                 // every pipe_gap-th operation waits for the previous frame (see enqueue_frame):
                                      // a wait on an event that has not completed costs the host several microseconds,
                                      // and the frame rate of a small network is bound by exactly that.  Networks of
                                      // few operations wait more often: a frame that waited for the end of the previous
                                      // one before its first kernel would overlap nothing
    long long frame_index = 0;
    int static_device = -1;   // >= 0: the workspace is that device's static array (cbinfer_create_static)
    bool initialised = false; // a frame has been processed since create/reset
    bool force_dense = false;
    bool broken = false;
    bool have_frame = false;
    bool lists_stale = false; // layers in selection mode have not had their index lists extracted for the last frame
    bool profiling = false;
    std::vector<EventPair> events;
    size_t events_used = 0;
    std::vector<double> prof_ms;
    std::vector<long long> prof_n;

    template <class T>
    T *at(size_t off) const
    {
        if (off == SIZE_MAX) return nullptr;
        if (off >= plan.o_set0 && off < plan.o_set0 + plan.set_bytes) off += (size_t)par * plan.set_bytes;
        return reinterpret_cast<T *>(ws + off);
    }
    bool pipelined() const { return plan.pipeline && !profiling; }
};

namespace {

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            s->broken = true;                                                                      \
            return fail(CBINFER_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(e_));           \
        }                                                                                          \
    } while (0)

// Hands the launch(es) of one step a pair of events that receive the kernel's own start and end
// time stamps (profiling on), or nothing.
struct StepTimer {
    EventPair *ep = nullptr;
    StepTimer(cbinfer_state *s, int layer, int step)
    {
        if (!s->profiling) return;
        if (s->events_used == s->events.size()) {
            EventPair p;
            if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) return;
            s->events.push_back(p);
        }
        ep = &s->events[s->events_used++];
        ep->layer = layer;
        ep->step = step;
    }
    cbk::Timing timing() const { return ep ? cbk::Timing{ep->a, ep->b} : cbk::Timing{}; }
};

int collect_profile(cbinfer_state *s)
{
    if (!s->profiling || s->events_used == 0) return CBINFER_OK;
    HIP_TRY(hipStreamSynchronize(s->work));
    for (size_t i = 0; i < s->events_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, s->events[i].a, s->events[i].b) == hipSuccess) {
            const size_t k = (size_t)s->events[i].layer * CBINFER_STEP_COUNT + s->events[i].step;
            s->prof_ms[k] += ms;
            s->prof_n[k] += 1;
        }
    }
    s->events_used = 0;
    return CBINFER_OK;
}

// Filter matrix K (Section 3) re-laid-out for the gather: row o, column k = (j*kw + i)*Cs + c,
// as float32 or bfloat16 (round to nearest even) bytes.
void build_filter_matrix(const Op &op, int dtype, const float *w, std::vector<unsigned char> &bytes)
{
    std::vector<float> wt((size_t)op.Mpad * op.Kpad, 0.0f);
    for (int o = 0; o < op.M; ++o)
        for (int c = 0; c < op.C; ++c)
            for (int j = 0; j < op.kh; ++j)
                for (int i = 0; i < op.kw; ++i)
                    wt[(size_t)o * op.Kpad + (size_t)(j * op.kw + i) * op.Cs + c] =
                        w[(((size_t)o * op.C + c) * op.kh + j) * op.kw + i];
    if (dtype == cbk::kBF16) {
        bytes.resize(wt.size() * 2);
        unsigned short *b = reinterpret_cast<unsigned short *>(bytes.data());
        for (size_t i = 0; i < wt.size(); ++i) b[i] = cbk::bf16_bits(wt[i]);
    } else {
        bytes.resize(wt.size() * 4);
        memcpy(bytes.data(), wt.data(), bytes.size());
    }
}

// One entry per 16-byte unit of a filter-matrix row: where its tap sits relative to the window origin.
void build_taps(const Op &op, int dtype, std::vector<int2> &taps)
{
    const int eu = cbk::elems_per_unit(dtype);
    taps.resize(op.Kpad / eu);
    for (int v = 0; v < op.Kpad / eu; ++v) {
        const int k = v * eu;
        int2 t;
        if (k < op.K) {
            const int tap = k / op.Cs, c = k - tap * op.Cs;
            const int j = tap / op.kw, i = tap - j * op.kw;
            t.x = (j * op.W + i) * op.pix_words + c / eu * 4;
            t.y = j | (i << 8) | (1 << 16);
        } else {
            t.x = 0;
            t.y = 0;
        }
        taps[v] = t;
    }
}

// Whether conv op l takes its change bitmap from the op that produces its input.
bool fuses_detection(const Plan &P, int l, bool force_dense)
{
    return l > 0 && !P.hold && !P.ops[l].dense && !P.ops[l].propagate && !force_dense;
}

// Whether conv op l runs no detection and takes the positions recomputed by the op before it as changed.
bool propagates(const Plan &P, int l, bool force_dense) { return l > 0 && P.ops[l].propagate && !force_dense; }

// The maps of convolution op l in a change-based frame.
struct LayerMaps {
    uint64_t *chg;   // changed input positions: one bit per pixel, or one byte when chg_bytes
    int chg_bytes;
    uint64_t *upd;   // output positions to recompute (the change map itself for a 1x1 layer without pooling)
    int upd_bytes;
    uint64_t *pool;  // pooled positions to recompute, nullptr without pooling
    bool identity;   // upd == chg: no dilation launch
    bool in_gemm;    // the multiplication kernel dilates chg itself and writes upd: no dilation launch,
                     // and the pooled bitmap is not filled in during the frame
};

LayerMaps layer_maps(const cbinfer_state *s, int l)
{
    const Plan &P = s->plan;
    const Op &op = P.ops[l];
    LayerMaps m;
    m.chg = s->at<uint64_t>(op.o_chg);
    m.chg_bytes = fuses_detection(P, l, s->force_dense) ? 1 : 0;
    if (propagates(P, l, s->force_dense)) {
        // the update map of the convolution before, carried through the pooling in between if any
        const Op &before = P.ops[l - 1];
        const int cl = before.kind == CBINFER_OP_CONV ? l - 1 : before.conv_before;
        const LayerMaps pm = layer_maps(s, cl);
        m.chg = before.kind == CBINFER_OP_CONV ? pm.upd : pm.pool;
        m.chg_bytes = before.kind == CBINFER_OP_CONV ? pm.upd_bytes : 0;
    }
    m.pool = op.pool_after >= 0 ? s->at<uint64_t>(op.o_pool) : nullptr;
    m.identity = op.kh == 1 && op.kw == 1 && op.stride == 1 && op.pad == 0 && !m.pool;
    m.upd = m.identity ? m.chg : s->at<uint64_t>(op.o_upd);
    m.upd_bytes = m.identity ? m.chg_bytes : 0;
    // a propagating layer behind this layer's pooling reads the pooled bitmap during the frame
    const bool pool_map_wanted = op.pool_after >= 0 && op.pool_after + 1 < (int)P.ops.size() &&
                                 propagates(P, op.pool_after + 1, s->force_dense);
    m.in_gemm = !m.identity && op.select && op.stride == 1 && op.kw <= 16 && op.kh <= 16 && !s->force_dense && !pool_map_wanted &&
                words_for((long long)P.S * op.H * op.Wo) <= cbk::gemm_select_max_words();
    return m;
}

// The three group-count arrays of op l (update map, change map, pooled map), one behind the other.
struct GroupCounts {
    int *upd, *chg, *pool;
};
GroupCounts group_counts(const cbinfer_state *s, int l)
{
    const Plan &P = s->plan;
    const Op &op = P.ops[l];
    const long long N = (long long)P.S * op.H * op.W, No = (long long)P.S * op.Ho * op.Wo;
    const size_t gstride = cbk::compact_group_count_bytes(words_for(std::max(N, No))) / sizeof(int);
    int *groups = s->at<int>(op.o_groups);
    return {groups, groups + gstride, groups + 2 * gstride};
}

// Dilation launch for op l: change map -> map of outputs to recompute (+ pooled positions).
// counted (optional) is set if the launch also left the maps' group counts for extract_lists.
hipError_t dilate_maps(const cbinfer_state *s, int l, const LayerMaps &m, bool *counted = nullptr,
                       const cbk::Timing &tm = cbk::Timing())
{
    const Plan &P = s->plan;
    const Op &op = P.ops[l];
    cbk::DilateGeom g;
    g.S = P.S; g.H = op.H; g.W = op.W; g.Ho = op.Ho; g.Wo = op.Wo;
    g.kh = op.kh; g.kw = op.kw; g.stride = op.stride; g.pad = op.pad;
    g.pool_k = 0; g.Hp = 0; g.Wp = 0;
    g.chg_bytes = m.chg_bytes;
    if (op.pool_after >= 0) {
        const Op &pp = P.ops[op.pool_after];
        g.pool_k = pp.kh; g.Hp = pp.Ho; g.Wp = pp.Wo;
    }
    if (counted) {
        const GroupCounts gc = group_counts(s, l);
        const cbk::DilateGroups dg = {gc.upd, gc.pool, gc.chg};
        *counted = cbk::dilate_counts(g) && (gc.pool != nullptr || !m.pool);
        return cbk::dilate(s->work, m.chg, m.upd, m.pool, g, &dg, tm);
    }
    return cbk::dilate(s->work, m.chg, m.upd, m.pool, g, nullptr, tm);
}

// Change-index extraction for op l (and the pooling op behind it): maps -> ascending lists and counts.
// counted: the dilation launch of this frame has left the group counts of all three maps.
hipError_t extract_lists(const cbinfer_state *s, int l, const LayerMaps &m, bool counted = false,
                         const cbk::Timing &tm = cbk::Timing())
{
    const Plan &P = s->plan;
    const Op &op = P.ops[l];
    const long long N = (long long)P.S * op.H * op.W, No = (long long)P.S * op.Ho * op.Wo;
    int *counts = s->at<int>(op.o_counts);
    const GroupCounts gc = group_counts(s, l);
    cbk::CompactJob jobs[3];
    int nj = 0;
    jobs[nj++] = {m.upd, m.upd_bytes, words_for(No), s->at<int>(op.o_ulist), counts + 1, gc.upd};
    jobs[nj++] = {m.chg, m.chg_bytes, words_for(N), s->at<int>(op.o_clist), counts + 0, gc.chg};
    if (m.pool) {
        const Op &pp = P.ops[op.pool_after];
        jobs[nj++] = {m.pool, 0, words_for((long long)P.S * pp.Ho * pp.Wo), s->at<int>(pp.o_ulist),
                      s->at<int>(pp.o_counts) + 1, gc.pool};
    }
    return cbk::compact(s->work, jobs, nj, counted, tm);
}


int enqueue_frame(cbinfer_state *s, const float *frame, float *out)
{
    const Plan &P = s->plan;
    const bool pipe = s->pipelined();
    const int slot = pipe ? (int)(s->frame_index & 1) : s->par, prev = slot ^ 1;
    hipStream_t st = pipe ? s->pstream[slot] : s->stream;
    if (pipe && hipStreamQuery(s->stream) != hipSuccess) {
        // whatever the caller's stream still does (to the frame buffer, say) comes first
        HIP_TRY(hipEventRecord(s->ev_in, s->stream));
        HIP_TRY(hipStreamWaitEvent(st, s->ev_in, 0));
    }
    s->par = slot;
    s->work = st;
    // An operation's kernels overwrite its stored output map, which the previous frame's kernels of
    // the operation behind it (at the end: the output copy) read; the first layer's detection
    // overwrites its stored input, which its own multiplication reads.  So before operation l this
    // frame's stream waits for the previous frame's operation l + 1 -- or for a later one: only every
    // gap-th operation waits, then for operation l + gap, which covers the operations up to the next
    // wait as well (both streams run their kernels in order).  Event n_ops stands for the output copy.
    // An event is recorded by the launch itself: the last kernel of an operation that somebody will
    // wait for hands it to the launch as its completion event.
    const int gap = s->pipe_gap, nops_ = (int)P.ops.size();
    auto after_previous = [&](int l) -> hipError_t {
        if (!pipe || !s->have_prev || l % gap != 0) return hipSuccess;
        return hipStreamWaitEvent(st, s->ev_op[prev][l + gap < nops_ ? l + gap : nops_], 0);
    };
    auto completion = [&](int ev, cbk::Timing tm) -> cbk::Timing {
        if (pipe && (ev == nops_ || (ev >= gap && ev % gap == 0))) tm.stop = s->ev_op[slot][ev];
        return tm;
    };
    const bool first = !s->initialised;
    s->lists_stale = false;
    const int S = P.S;
    int *iota = s->at<int>(P.o_iota);
    int *consts = s->at<int>(P.o_const);
    const int nops = (int)P.ops.size();

    for (int l = 0; l < nops; ++l) {
        const Op &op = P.ops[l];
        if (op.kind == CBINFER_OP_CONV) {
            const int N = op.H * op.W, No = op.Ho * op.Wo;
            const void *x = nullptr;
            const int eu = cbk::elems_per_unit(P.dtype);
            void *ref = s->at<void>(op.o_ref);
            int *counts = s->at<int>(op.o_counts);
            const bool all = first || op.dense || s->force_dense;
            // A layer fed by a stored map finds its changes while that map is updated (the op
            // before it compares each new value with the one it replaces), unless it holds its
            // reference or runs densely.
            const bool fused_in = fuses_detection(P, l, s->force_dense);
            // --- change detection (also turns the planar frame into a map for layer 0)
            if (l == 0) {
                HIP_TRY(after_previous(0));
                StepTimer t(s, l, CBINFER_STEP_DETECT);
                const int hold = (P.hold && !s->force_dense) ? 1 : 0;
                // the same launch zeroes the byte change maps that this frame's kernels fill in
                uint64_t *flags = s->force_dense ? nullptr : s->at<uint64_t>(P.o_flags);
                HIP_TRY(cbk::detect_frame(st, frame, ref, s->at<void>(op.o_cur), s->at<uint64_t>(op.o_chg), op.C,
                                          op.Cs / eu, N, S, op.tau, hold, all ? 1 : 0, P.dtype,
                                          op.pix_words == op.C && op.C % 4 != 0, flags, P.flag_words, t.timing()));
                x = hold ? s->at<void>(op.o_cur) : ref;
            } else {
                x = s->at<void>(P.ops[l - 1].o_out);
                if (!s->force_dense && !fused_in && !op.propagate) {
                    StepTimer t(s, l, CBINFER_STEP_DETECT);
                    HIP_TRY(cbk::detect_map(st, x, ref, s->at<uint64_t>(op.o_chg), op.Cs / eu, S * N, op.tau,
                                            P.hold ? 1 : 0, all ? 1 : 0, P.dtype, t.timing()));
                }
            }
            if (l > 0) HIP_TRY(after_previous(l));
            const int *ulist = iota;
            const int *ucount = consts + 2 * l;
            const uint64_t *sel_map = nullptr;
            int sel_bytes = 0, sel_dilate = 0;
            if (!s->force_dense) {
                const LayerMaps m = layer_maps(s, l);
                bool counted = false;
                if (!m.identity && !m.in_gemm) {
                    StepTimer t(s, l, CBINFER_STEP_DILATE);
                    HIP_TRY(dilate_maps(s, l, m, op.select ? nullptr : &counted, t.timing()));
                }
                if (op.select) {
                    sel_map = m.in_gemm ? m.chg : m.upd;
                    sel_bytes = m.in_gemm ? m.chg_bytes : m.upd_bytes;
                    sel_dilate = m.in_gemm ? 1 : 0;
                    ulist = nullptr;
                    ucount = nullptr;
                    s->lists_stale = true;
                } else {
                    StepTimer t(s, l, CBINFER_STEP_COMPACT);
                    HIP_TRY(extract_lists(s, l, m, counted, t.timing()));
                    ulist = s->at<int>(op.o_ulist);
                    ucount = counts + 1;
                }
            }
            // --- gathered matrix generation + multiplication + output update
            cbk::GemmArgs a;
            a.dtype = P.dtype;
            a.x = x;
            a.wt = s->at<void>(op.o_wt);
            a.bias = s->at<float>(op.o_bias);
            a.taps = s->at<int2>(op.o_taps);
            a.list = ulist;
            a.count = ucount;
            a.sel_map = sel_map;
            a.sel_bytes = sel_bytes;
            a.sel_words = sel_map ? words_for((long long)S * No) : 0;
            a.sel_dilate = sel_dilate;
            a.sel_in_words = words_for((long long)S * N);
            a.upd_out = s->at<uint64_t>(op.o_upd);
            a.kh = op.kh; a.kw = op.kw; a.S = S;
            a.out = s->at<void>(op.o_out);
            a.N = N; a.H = op.H; a.W = op.W; a.No = No; a.Wo = op.Wo;
            a.stride = op.stride; a.pad = op.pad; a.pix_words = op.pix_words; a.Kpad = op.Kpad;
            a.zero_word = S * N * op.pix_words;
            a.M = op.M; a.Mpad = op.Mpad; a.Ms = op.Ms; a.relu = op.relu;
            a.max_pixels = S * No;
            a.partial = s->at<float>(P.o_partial);
            a.tickets = s->at<int>(P.o_tickets);
            a.grid = op.gemm_grid;
            a.next_flags = nullptr;
            a.next_tau = 0.f;
            a.next_force = first ? 1 : 0;
            if (l + 1 < nops && P.ops[l + 1].kind == CBINFER_OP_CONV && fuses_detection(P, l + 1, s->force_dense)) {
                a.next_flags = s->at<unsigned char>(P.ops[l + 1].o_chg);
                a.next_tau = P.ops[l + 1].tau;
            }
            cbk::gemm_set_divisors(a);
            {
                StepTimer t(s, l, CBINFER_STEP_GEMM);
                HIP_TRY(cbk::gemm_gather(st, a, completion(l, t.timing())));
            }
        } else {
            HIP_TRY(after_previous(l));
            const Op &cv = P.ops[op.conv_before];
            const int Np = op.Ho * op.Wo;
            const int *plist = s->force_dense ? iota : s->at<int>(op.o_ulist);
            const int *pcount = s->force_dense ? consts + 2 * l : s->at<int>(op.o_counts) + 1;
            unsigned char *next_flags = nullptr;
            float next_tau = 0.f;
            if (l + 1 < nops && P.ops[l + 1].kind == CBINFER_OP_CONV && fuses_detection(P, l + 1, s->force_dense)) {
                next_flags = s->at<unsigned char>(P.ops[l + 1].o_chg);
                next_tau = P.ops[l + 1].tau;
            }
            StepTimer t(s, l, CBINFER_STEP_POOL);
            if (cv.select && !s->force_dense) {
                // the pooled bitmap, or (when the multiplication kernel derived the update map itself)
                // the update bitmap of the convolution, tested window by window
                const LayerMaps cm = layer_maps(s, op.conv_before);
                HIP_TRY(cbk::pool_masked(st, cm.in_gemm ? cm.upd : cm.pool, cm.in_gemm ? 1 : 0, S * Np,
                                         s->at<void>(cv.o_out), s->at<void>(op.o_out),
                                         op.Ms / cbk::elems_per_unit(P.dtype), op.kh, cv.Wo, cv.Ho * cv.Wo, op.Wo, Np,
                                         next_flags, next_tau, first ? 1 : 0, P.dtype, completion(l, t.timing())));
            }
            else
                HIP_TRY(cbk::pool_sparse(st, plist, pcount, S * Np, s->at<void>(cv.o_out), s->at<void>(op.o_out),
                                         op.Ms / cbk::elems_per_unit(P.dtype), op.kh, cv.Wo, cv.Ho * cv.Wo, op.Wo, Np,
                                         next_flags, next_tau, first ? 1 : 0, P.dtype, completion(l, t.timing())));
        }
    }
    const Op &last = P.ops.back();
    {
        StepTimer t(s, nops - 1, CBINFER_STEP_OUTPUT);
        HIP_TRY(cbk::map_to_planar(st, s->at<void>(last.o_out), out, last.M, last.Ms / cbk::elems_per_unit(P.dtype),
                                   last.Ho * last.Wo, S, P.dtype, completion(nops, t.timing())));
    }
    if (pipe) {
        s->have_prev = true;
        ++s->frame_index;
    }
    s->initialised = true;
    s->have_frame = true;
    return collect_profile(s);
}

} // namespace

extern "C" {

const char *cbinfer_last_error(void) { return g_err.c_str(); }

size_t cbinfer_workspace_bytes(const cbinfer_network *net)
{
    Plan P;
    if (make_plan(net, 0.0f, false, P) != CBINFER_OK) return 0;
    return P.bytes;
}

static void release_pipeline(cbinfer_state *s)
{
    for (int i = 0; i < 2; ++i) {
        for (hipEvent_t e : s->ev_op[i])
            if (e) (void)hipEventDestroy(e);
        s->ev_op[i].clear();
        if (s->pstream[i]) (void)hipStreamDestroy(s->pstream[i]);
        s->pstream[i] = nullptr;
    }
    if (s->ev_in) (void)hipEventDestroy(s->ev_in);
    s->ev_in = nullptr;
}

// Common part of cbinfer_create and cbinfer_create_static.  ws: device memory for the whole
// workspace (P.bytes, 256-byte aligned) or nullptr to allocate it here.
static cbinfer_state *create_state(const cbinfer_network *net, const Plan &P, char *ws, int static_device)
{
    cbinfer_state *s = new cbinfer_state();
    s->plan = P;
    s->stream = reinterpret_cast<hipStream_t>(net->stream);
    s->work = s->stream;
    s->static_device = static_device;
    if (ws) {
        s->ws = ws;
    } else {
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, P.bytes);
        if (e != hipSuccess) {
            fail(CBINFER_ENOMEM, "hipMalloc of %zu bytes failed: %s", P.bytes, hipGetErrorString(e));
            delete s;
            return nullptr;
        }
        s->ws = static_cast<char *>(p);
        s->owns_ws = true;
    }
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            s->plan.compute_units = cus < kMaxGemmGrid ? cus : kMaxGemmGrid;
    }
    for (Op &op : s->plan.ops) {
        if (op.kind != CBINFER_OP_CONV) continue;
        cbk::GemmArgs a{};
        a.dtype = P.dtype;
        a.M = op.M; a.Mpad = op.Mpad; a.Kpad = op.Kpad;
        a.max_pixels = P.S * op.Ho * op.Wo;
        op.gemm_grid = cbk::gemm_grid(a, s->plan.compute_units);
    }
    s->prof_ms.assign(P.ops.size() * CBINFER_STEP_COUNT, 0.0);
    s->prof_n.assign(P.ops.size() * CBINFER_STEP_COUNT, 0);

    auto setup = [&]() -> int {
        HIP_TRY(cbk::gemm_prepare());
        if (P.pipeline) {
            // two streams of the library's own (default priority) and the events that order frames in flight
            HIP_TRY(hipEventCreateWithFlags(&s->ev_in, hipEventDisableTiming));
            for (int i = 0; i < 2; ++i) {
                HIP_TRY(hipStreamCreateWithFlags(&s->pstream[i], hipStreamNonBlocking));
                s->pipe_gap = P.ops.size() >= 12 ? 4 : (P.ops.size() >= 6 ? 3 : (P.ops.size() >= 4 ? 2 : 1));
                s->ev_op[i].assign(P.ops.size() + 1, nullptr);
                for (hipEvent_t &e : s->ev_op[i]) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            }
        }
        // everything starts at zero: stored maps and their zero units, change maps, counters, tickets
        // (the static workspace keeps whatever the state before this one left in it)
        HIP_TRY(hipMemsetAsync(s->ws, 0, P.bytes, s->stream));
        std::vector<unsigned char> wt;
        std::vector<float> bias;
        std::vector<int2> taps;
        std::vector<int> consts(P.ops.size() * 2, 0);
        for (size_t l = 0; l < P.ops.size(); ++l) {
            const Op &op = P.ops[l];
            consts[2 * l] = P.S * op.Ho * op.Wo;
            if (op.kind != CBINFER_OP_CONV) continue;
            const cbinfer_layer &L = net->layers[l];
            build_filter_matrix(op, P.dtype, static_cast<const float *>(L.weight), wt);
            bias.assign(op.Mpad, 0.0f);
            if (L.bias)
                for (int o = 0; o < op.M; ++o) bias[o] = L.bias[o];
            build_taps(op, P.dtype, taps);
            // the staging vectors are reused for the next layer: wait for the copies first
            HIP_TRY(hipMemcpyAsync(s->at<void>(op.o_wt), wt.data(), wt.size(), hipMemcpyHostToDevice, s->stream));
            HIP_TRY(hipMemcpyAsync(s->at<float>(op.o_bias), bias.data(), bias.size() * 4, hipMemcpyHostToDevice, s->stream));
            HIP_TRY(hipMemcpyAsync(s->at<int2>(op.o_taps), taps.data(), taps.size() * sizeof(int2), hipMemcpyHostToDevice, s->stream));
            HIP_TRY(hipStreamSynchronize(s->stream));
        }
        HIP_TRY(hipMemcpyAsync(s->at<int>(P.o_const), consts.data(), consts.size() * 4, hipMemcpyHostToDevice, s->stream));
        HIP_TRY(cbk::fill_iota(s->stream, s->at<int>(P.o_iota), P.iota_len));
        HIP_TRY(hipStreamSynchronize(s->stream));
        return CBINFER_OK;
    };
    if (setup() != CBINFER_OK) {
        release_pipeline(s);
        if (s->owns_ws) (void)hipFree(s->ws);
        delete s;
        return nullptr;
    }
    return s;
}

cbinfer_state *cbinfer_create(const cbinfer_network *net, float threshold)
{
    Plan P;
    if (make_plan(net, threshold, true, P) != CBINFER_OK) return nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
        fail(CBINFER_EDEVICE, "no HIP device available (this library has no CPU path)");
        return nullptr;
    }
    if (net->workspace) {
        if (reinterpret_cast<uintptr_t>(net->workspace) % kAlign) {
            fail(CBINFER_EINVAL, "workspace must be %zu-byte aligned", kAlign);
            return nullptr;
        }
        if (net->workspace_bytes < P.bytes) {
            fail(CBINFER_ENOMEM, "workspace has %zu bytes, %zu needed", net->workspace_bytes, P.bytes);
            return nullptr;
        }
    }
    return create_state(net, P, static_cast<char *>(net->workspace), -1);
}

// ---- the entry point that allocates no device memory ------------------------------------------
// All state and scratch of a network (stored maps, change maps, index lists, filter matrices, the
// partial-accumulator slabs and ticket counters of the multiplication kernel) in a device array
// that is part of the library's code object: every GPU the library is loaded on holds one copy of
// it, at an address of its own, from module load until the process ends.
static __device__ __align__(256) unsigned char scratch[CBINFER_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
char *g_scratch_ptr[kMaxDevices] = {};    // device address of `scratch` on each device, once looked up
bool g_scratch_in_use[kMaxDevices] = {};  // a live state occupies that device's array
} // namespace

cbinfer_state *cbinfer_create_static(const cbinfer_network *net, float threshold)
{
    Plan P;
    if (make_plan(net, threshold, true, P) != CBINFER_OK) return nullptr;
    if (P.bytes > (size_t)CBINFER_STATIC_WORKSPACE_BYTES) {
        fail(CBINFER_ENOMEM,
             "this network needs %zu bytes of state and scratch; the static workspace holds %zu "
             "(use cbinfer_create with a caller workspace)",
             P.bytes, (size_t)CBINFER_STATIC_WORKSPACE_BYTES);
        return nullptr;
    }
    int ndev = 0, dev = -1;
    hipError_t de = hipGetDeviceCount(&ndev);
    if (de != hipSuccess || ndev < 1) {
        fail(CBINFER_EDEVICE, "no HIP device available (this library has no CPU path): hipGetDeviceCount says %s, %d devices",
             hipGetErrorString(de), ndev);
        return nullptr;
    }
    if ((de = hipGetDevice(&dev)) != hipSuccess) {
        fail(CBINFER_EDEVICE, "no current HIP device: hipGetDevice says %s", hipGetErrorString(de));
        return nullptr;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        fail(CBINFER_EUNSUPPORTED, "device ordinal %d is beyond the %d devices the static workspace is tracked for", dev,
             kMaxDevices);
        return nullptr;
    }
    char *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (g_scratch_in_use[dev]) {
            fail(CBINFER_ESTATE, "the static workspace of device %d is in use by a state that has not been destroyed", dev);
            return nullptr;
        }
        if (!g_scratch_ptr[dev]) {
            // `scratch` names the array for the host compiler only; its device address (one per
            // device) has to be asked for, with that device current
            void *p = nullptr;
            const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) {
                fail(CBINFER_EDEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
                return nullptr;
            }
            g_scratch_ptr[dev] = static_cast<char *>(p);
        }
        ptr = g_scratch_ptr[dev];
        g_scratch_in_use[dev] = true;
    }
    cbinfer_state *s = create_state(net, P, ptr, dev);
    if (!s) {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        g_scratch_in_use[dev] = false;
    }
    return s;
}

size_t cbinfer_static_workspace_bytes(void) { return (size_t)CBINFER_STATIC_WORKSPACE_BYTES; }

int cbinfer_process_frame(cbinfer_state *s, const void *frame_dev, void *out_dev)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (!frame_dev || !out_dev) return fail(CBINFER_EINVAL, "frame and output pointers must not be NULL");
    if (s->broken) return fail(CBINFER_EDEVICE, "a previous HIP call failed; destroy this state");
    return enqueue_frame(s, static_cast<const float *>(frame_dev), static_cast<float *>(out_dev));
}

int cbinfer_flush(cbinfer_state *s)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (s->broken) return fail(CBINFER_EDEVICE, "a previous HIP call failed; destroy this state");
    if (s->plan.pipeline && s->have_prev) {
        const int last = (int)((s->frame_index + 1) & 1); // slot of the frame enqueued last
        HIP_TRY(hipStreamWaitEvent(s->stream, s->ev_op[last][s->plan.ops.size()], 0));
    }
    return CBINFER_OK;
}

int cbinfer_reset(cbinfer_state *s)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    s->initialised = false;
    return CBINFER_OK;
}

void cbinfer_destroy(cbinfer_state *s)
{
    if (!s) return;
    for (int i = 0; i < 2; ++i)
        if (s->pstream[i]) (void)hipStreamSynchronize(s->pstream[i]);
    (void)hipStreamSynchronize(s->stream);
    release_pipeline(s);
    for (auto &e : s->events) {
        if (e.a) (void)hipEventDestroy(e.a);
        if (e.b) (void)hipEventDestroy(e.b);
    }
    if (s->owns_ws && s->ws) (void)hipFree(s->ws);
    if (s->static_device >= 0) {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        g_scratch_in_use[s->static_device] = false;
    }
    delete s;
}

// Waits until no frame is in flight any more (and nothing else on the caller's stream).
static int drain(cbinfer_state *s)
{
    for (int i = 0; i < 2; ++i)
        if (s->pstream[i]) HIP_TRY(hipStreamSynchronize(s->pstream[i]));
    HIP_TRY(hipStreamSynchronize(s->stream));
    s->have_prev = false;
    return CBINFER_OK;
}

// Layers in selection mode keep their maps and skip index extraction in the frame itself; the
// lists and counts of the last frame are extracted here, the first time they are asked for.
static int refresh_lists(cbinfer_state *s)
{
    if (!s->lists_stale) return CBINFER_OK;
    for (int l = 0; l < (int)s->plan.ops.size(); ++l) {
        const Op &op = s->plan.ops[l];
        if (op.kind != CBINFER_OP_CONV || !op.select) continue;
        const LayerMaps m = layer_maps(s, l);
        // the frame skipped the dilation kernel: the pooled bitmap has not been filled in yet
        if (m.in_gemm && m.pool) HIP_TRY(dilate_maps(s, l, m));
        HIP_TRY(extract_lists(s, l, m));
    }
    s->lists_stale = false;
    return CBINFER_OK;
}

int cbinfer_set_mode(cbinfer_state *s, int force_dense)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (!s->broken && s->have_frame) {
        int rc = drain(s);
        if (rc == CBINFER_OK) rc = refresh_lists(s); // under the mode the last frame ran in
        if (rc) return rc;
    }
    s->force_dense = force_dense != 0;
    s->initialised = false;
    return CBINFER_OK;
}

int cbinfer_layer_shape(cbinfer_state *s, int layer, int32_t *c, int32_t *h, int32_t *w)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (layer < 0 || layer >= (int)s->plan.ops.size()) return fail(CBINFER_EINVAL, "layer %d out of range", layer);
    const Op &op = s->plan.ops[layer];
    if (c) *c = op.M;
    if (h) *h = op.Ho;
    if (w) *w = op.Wo;
    return CBINFER_OK;
}

static int check_query(cbinfer_state *s, int layer)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (layer < 0 || layer >= (int)s->plan.ops.size()) return fail(CBINFER_EINVAL, "layer %d out of range", layer);
    if (s->broken) return fail(CBINFER_EDEVICE, "a previous HIP call failed; destroy this state");
    if (!s->have_frame) return fail(CBINFER_ESTATE, "no frame has been processed yet");
    return CBINFER_OK;
}

int cbinfer_layer_counts(cbinfer_state *s, int layer, int64_t *n_changed, int64_t *n_update)
{
    int rc = check_query(s, layer);
    if (rc) return rc;
    if ((rc = drain(s)) != CBINFER_OK || (rc = refresh_lists(s)) != CBINFER_OK) return rc;
    const Op &op = s->plan.ops[layer];
    int c[2] = {0, 0};
    if (s->force_dense) {
        c[0] = op.kind == CBINFER_OP_CONV ? s->plan.S * op.H * op.W : -1;
        c[1] = s->plan.S * op.Ho * op.Wo;
    } else {
        HIP_TRY(hipStreamSynchronize(s->work));
        HIP_TRY(hipMemcpy(c, s->at<int>(op.o_counts), 8, hipMemcpyDeviceToHost));
        if (op.kind != CBINFER_OP_CONV) c[0] = -1;
    }
    if (n_changed) *n_changed = c[0];
    if (n_update) *n_update = c[1];
    return CBINFER_OK;
}

int cbinfer_read_list(cbinfer_state *s, int layer, int which, int32_t *host, int64_t cap, int64_t *n)
{
    int rc = check_query(s, layer);
    if (rc) return rc;
    if (which != CBINFER_LIST_CHANGED && which != CBINFER_LIST_UPDATE && which != CBINFER_LIST_POOLED)
        return fail(CBINFER_EINVAL, "unknown list %d", which);
    if (which == CBINFER_LIST_POOLED) {
        // the pooled positions behind a convolution: the update list of the pooling op that follows it
        const Op &cv = s->plan.ops[layer];
        if (cv.kind != CBINFER_OP_CONV || cv.pool_after < 0)
            return fail(CBINFER_EINVAL, "layer %d is not a convolution directly followed by pooling", layer);
        layer = cv.pool_after;
        which = CBINFER_LIST_UPDATE;
    }
    const Op &op = s->plan.ops[layer];
    if (which == CBINFER_LIST_CHANGED && op.kind != CBINFER_OP_CONV)
        return fail(CBINFER_EINVAL, "layer %d is a pooling layer and has no changed-input list", layer);
    if (cap < 0 || (cap > 0 && !host)) return fail(CBINFER_EINVAL, "bad host buffer");
    if ((rc = drain(s)) != CBINFER_OK || (rc = refresh_lists(s)) != CBINFER_OK) return rc;
    HIP_TRY(hipStreamSynchronize(s->work));
    int count = 0;
    const int *src = nullptr;
    if (s->force_dense) {
        count = which == CBINFER_LIST_CHANGED ? s->plan.S * op.H * op.W : s->plan.S * op.Ho * op.Wo;
        src = s->at<int>(s->plan.o_iota);
    } else {
        HIP_TRY(hipMemcpy(&count, s->at<int>(op.o_counts) + (which == CBINFER_LIST_CHANGED ? 0 : 1), 4,
                          hipMemcpyDeviceToHost));
        src = which == CBINFER_LIST_CHANGED ? s->at<int>(op.o_clist) : s->at<int>(op.o_ulist);
    }
    if (n) *n = count;
    const int64_t m = count < cap ? count : cap;
    if (m > 0) HIP_TRY(hipMemcpy(host, src, (size_t)m * 4, hipMemcpyDeviceToHost));
    return CBINFER_OK;
}

int cbinfer_read_map(cbinfer_state *s, int layer, int which, float *host, size_t count)
{
    int rc = check_query(s, layer);
    if (rc) return rc;
    if (!host) return fail(CBINFER_EINVAL, "host buffer is NULL");
    const Op &op = s->plan.ops[layer];
    int C, Cs, HW;
    const void *src;
    if (which == CBINFER_MAP_REFERENCE) {
        if (op.kind != CBINFER_OP_CONV) return fail(CBINFER_EINVAL, "layer %d has no stored previous input", layer);
        if (s->force_dense && layer > 0) return fail(CBINFER_ESTATE, "dense mode keeps no previous input for layer %d", layer);
        C = op.C; Cs = op.pix_words * 4 / cbk::elem_bytes(s->plan.dtype); HW = op.H * op.W;
        // a layer that keeps no copy of its own: its previous input is the stored map that feeds it
        src = op.o_ref != SIZE_MAX ? s->at<void>(op.o_ref) : s->at<void>(s->plan.ops[layer - 1].o_out);
    } else if (which == CBINFER_MAP_OUTPUT) {
        C = op.M; Cs = op.Ms; HW = op.Ho * op.Wo;
        src = s->at<void>(op.o_out);
    } else {
        return fail(CBINFER_EINVAL, "unknown map %d", which);
    }
    const size_t need = (size_t)s->plan.S * C * HW;
    if (count != need) return fail(CBINFER_EINVAL, "map has %zu values, buffer holds %zu", need, count);
    const size_t n_el = (size_t)s->plan.S * HW * Cs;
    if ((rc = drain(s)) != CBINFER_OK) return rc;
    if (s->plan.dtype == cbk::kBF16) {
        std::vector<unsigned short> tmp(n_el);
        HIP_TRY(hipMemcpy(tmp.data(), src, n_el * 2, hipMemcpyDeviceToHost));
        for (int st = 0; st < s->plan.S; ++st)
            for (int c = 0; c < C; ++c)
                for (int p = 0; p < HW; ++p)
                    host[((size_t)st * C + c) * HW + p] = cbk::bf16_value(tmp[((size_t)st * HW + p) * Cs + c]);
    } else {
        std::vector<float> tmp(n_el);
        HIP_TRY(hipMemcpy(tmp.data(), src, n_el * 4, hipMemcpyDeviceToHost));
        for (int st = 0; st < s->plan.S; ++st)
            for (int c = 0; c < C; ++c)
                for (int p = 0; p < HW; ++p)
                    host[((size_t)st * C + c) * HW + p] = tmp[((size_t)st * HW + p) * Cs + c];
    }
    return CBINFER_OK;
}

int cbinfer_set_profiling(cbinfer_state *s, int enable)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (s->broken) return fail(CBINFER_EDEVICE, "a previous HIP call failed; destroy this state");
    if (drain(s) != CBINFER_OK) return CBINFER_EDEVICE;
    s->profiling = enable != 0;
    s->events_used = 0;
    std::fill(s->prof_ms.begin(), s->prof_ms.end(), 0.0);
    std::fill(s->prof_n.begin(), s->prof_n.end(), 0);
    return CBINFER_OK;
}

int cbinfer_read_profile(cbinfer_state *s, int layer, int step, double *ms_total, int64_t *launches)
{
    if (!s) return fail(CBINFER_EINVAL, "state is NULL");
    if (layer < 0 || layer >= (int)s->plan.ops.size()) return fail(CBINFER_EINVAL, "layer %d out of range", layer);
    if (step < 0 || step >= CBINFER_STEP_COUNT) return fail(CBINFER_EINVAL, "step %d out of range", step);
    const size_t k = (size_t)layer * CBINFER_STEP_COUNT + step;
    if (ms_total) *ms_total = s->prof_ms[k];
    if (launches) *launches = s->prof_n[k];
    return CBINFER_OK;
}

} // extern "C"
