// One worker's SGD iteration with the turn-based, barrier-free schedule (section 2.3, Fig. 3).
//
// The compute stream runs forward 1..L, the loss, and backward L..1.  As soon as the local
// gradient of layer l is complete an event is recorded; the update stream waits for it and runs
// that layer's (K+1)-buffer gradient sum + model update while the compute stream continues with
// layer l-1 -- the paper's overlap of the reduction/update of one layer with the gradient
// computation of the layers below it.  "Finalize" is per layer as well: the next iteration's
// forward of layer l waits only on the event of layer l's own update, so there is no device-wide
// synchronisation anywhere (design principle 2, section 2.2).  Small layers share update launches
// (and with them events): up to eight of them, or a million parameters, per launch.
//
// Within a layer's turn backward-data and backward-weight are independent and run side by side
// (backward-weight on a third stream owned by the net); the update waits for both, because it
// overwrites the model that backward-data still reads.
#include <atomic>
#include <new>
#include <vector>
#include "cg_internal.h"

// How nets created from now on run an LRN layer followed by a max-pool: bit 0 = forward as one
// kernel, bit 1 = backward as one kernel.  Forward fused is the default; the fused backward is
// built and tested but bound by its instruction count, not by memory, and slower than the two
// separate kernels (measured), so it runs only when asked for.
static std::atomic<int> g_fuse_lrn_pool{1};
extern "C" int cg_debug_fuse_lrn_pool(int mode)
{
    if (mode < 0 || mode > 3 || mode == 2) return CG_EINVAL;     // backward fused needs forward fused
    g_fuse_lrn_pool.store(mode, std::memory_order_relaxed);
    return CG_OK;
}

struct cg_net {
    struct Layer {
        cg_layer_desc d;
        int inC = 0, inH = 0, inW = 0;        // shape of inputs[0]
        int C = 0, H = 0, W = 0;              // output shape
        cg_conv_desc conv{};                  // completed descriptor (CONV)
        size_t act_off = 0, grad_off = 0, aux_off = 0;   // float offsets into the workspace
        size_t out_elems = 0, aux_elems = 0;
        long long n_params = 0, n_weights = 0;
        float *w = nullptr, *v = nullptr, *g = nullptr;
        std::vector<const float *> peers;
        bool bound = false;
        hipEvent_t ev_grad = nullptr, ev_upd = nullptr;
        hipEvent_t ev_dy = nullptr, ev_bd = nullptr;   // gradient of the output complete / backward-data done
        bool upd_pending = false;             // an update of this layer was enqueued by a previous step
        hipEvent_t upd_event = nullptr;       // the event that update completes with: this layer's ev_upd, or that of
                                              // the last layer of the launch the update went out with
        bool grad_written = false;            // per step: has anything been written to this layer's gradient?
        bool needs_grad = false;              // false when no parameter lies upstream of this output
        // A rectifier that is the only consumer of a convolution or fully-connected layer is folded
        // into that layer's store: the producer (fused_relu) writes max(., 0) and the rectifier
        // (alias_of = producer) shares its output buffer and launches nothing in forward.  Its
        // backward needs only the sign, which the rectified output still carries.
        bool fused_relu = false;
        int alias_of = -1;
        // Backward of a rectifier whose only consumer is a convolution, fully-connected, LRN,
        // max-pool or dropout layer is folded into that consumer's backward kernel, which gates its
        // result with the rectifier's output and writes the gradient of the rectifier's INPUT: the
        // gradient with respect to the rectifier's output is never materialised (bwd_folded), and
        // the consumer knows the rectifier by gate_from.
        bool bwd_folded = false;
        int gate_from = -1;
        // A convolution whose folded rectifier feeds nothing but one concat writes straight into its
        // channel slice of the concat's output (out_img_stride = elements between images there; its
        // and the rectifier's act_off point at the slice), and the concat's backward gates the slice of
        // its gradient with that output on the way to the convolution's gradient (the rectifier is
        // bwd_folded with in_concat = the concat layer).
        long long out_img_stride = 0;
        int in_concat = -1;
        // An LRN layer whose only consumer is a max-pool runs fused with it (fused_pool = the pool,
        // the pool's fused_lrn = the LRN): forward at the pool's place, from the LRN's input straight
        // to the pooled output and the winners; backward at the LRN's place, from the pool's gradient
        // and winners straight to the gradient of the LRN's input.  The LRN's output and the gradient
        // with respect to it are never written.
        int fused_pool = -1, fused_lrn = -1;
        bool fused_pool_bwd = false;          // (LRN layer) backward fused as well
        // (CONV) room for the rearranged copies of the filters that forward and backward-data multiply
        // with; all of a net's copies are made by one or a few launches at the start of an iteration
        size_t prep_fwd_off = 0, prep_bd_off = 0;
        const float *prep_fwd = nullptr, *prep_bd = nullptr;      // per step: the copy, or null where the pass reads w itself
    };

    int B = 0, C = 0, H = 0, W = 0;
    std::vector<Layer> layers;
    size_t scratch_off = 0, scratch_bytes = 0;   // kernel scratch (filter copies, split-K partials): two regions of
                                                 // scratch_bytes, one per stream that launches matrix kernels
    hipStream_t wgrad_stream = nullptr;          // backward-weight passes run here, beside backward-data
    hipEvent_t ev_join = nullptr;                // tail of the update stream (CG_STEP_JOIN)
    size_t loss_off = 0;                         // B floats of per-sample loss
    size_t ws_floats = 0;
};

namespace {

using namespace cg;
using Layer = cg_net::Layer;

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

void in_shape(const cg_net &net, int src, int *C, int *H, int *W)
{
    if (src < 0) { *C = net.C; *H = net.H; *W = net.W; }
    else { *C = net.layers[src].C; *H = net.layers[src].H; *W = net.layers[src].W; }
}

}  // namespace

extern "C" int cg_net_create(const cg_layer_desc *descs, int L, int B, int C, int H, int W, cg_net **out)
{
    if (!descs || !out || L <= 0 || B <= 0 || C <= 0 || H <= 0 || W <= 0) return CG_EINVAL;
    cg_net *net = new (std::nothrow) cg_net;
    if (!net) return CG_EINVAL;
    net->B = B; net->C = C; net->H = H; net->W = W;
    net->layers.resize(L);
    size_t off = 0, scratch = 0;
    int rc = CG_OK;
    for (int i = 0; i < L && rc == CG_OK; ++i) {
        Layer &ly = net->layers[i];
        ly.d = descs[i];
        const cg_layer_desc &d = ly.d;
        if (d.n_inputs < 1 || d.n_inputs > 4 || (d.kind != CG_LAYER_CONCAT && d.n_inputs != 1)) { rc = CG_EINVAL; break; }
        for (int k = 0; k < d.n_inputs; ++k)
            if (d.inputs[k] < -1 || d.inputs[k] >= i) rc = CG_EINVAL;      // producers come first
        if (rc) break;
        in_shape(*net, d.inputs[0], &ly.inC, &ly.inH, &ly.inW);
        ly.needs_grad = false;
        for (int k = 0; k < d.n_inputs; ++k)
            if (d.inputs[k] >= 0 && (net->layers[d.inputs[k]].needs_grad)) ly.needs_grad = true;
        switch (d.kind) {
        case CG_LAYER_CONV: {
            ly.conv = d.conv;
            ly.conv.N = B; ly.conv.C = ly.inC; ly.conv.H = ly.inH; ly.conv.W = ly.inW;
            int OH, OW;
            rc = conv_check(&ly.conv, &OH, &OW);
            if (rc) break;
            ly.C = ly.conv.M; ly.H = OH; ly.W = OW;
            ly.n_weights = (long long)ly.conv.M * (ly.inC / ly.conv.groups) * ly.conv.KH * ly.conv.KW;
            ly.n_params = ly.n_weights + ly.conv.M;
            for (int pass = 0; pass < 3; ++pass) {
                const size_t sb = conv_ws_bytes(ly.conv, pass);
                if (sb > scratch) scratch = sb;
            }
            ly.needs_grad = true;
            break;
        }
        case CG_LAYER_FC:
            if (d.fc_out <= 0) { rc = CG_EINVAL; break; }
            ly.C = d.fc_out; ly.H = ly.W = 1;
            ly.n_weights = (long long)d.fc_out * ly.inC * ly.inH * ly.inW;
            ly.n_params = ly.n_weights + d.fc_out;
            if (ly.n_weights >= (1ll << 29)) rc = CG_EUNSUPPORTED;
            for (int pass = 0; pass < 3; ++pass) {
                const size_t sb = fc_ws_bytes(B, ly.inC * ly.inH * ly.inW, d.fc_out, pass);
                if (sb > scratch) scratch = sb;
            }
            ly.needs_grad = true;
            break;
        case CG_LAYER_RELU: case CG_LAYER_DROPOUT:
            ly.C = ly.inC; ly.H = ly.inH; ly.W = ly.inW;
            if (d.kind == CG_LAYER_DROPOUT && !(d.drop_p >= 0.f && d.drop_p < 1.f)) rc = CG_EINVAL;
            break;
        case CG_LAYER_LRN:
            ly.C = ly.inC; ly.H = ly.inH; ly.W = ly.inW;
            if (d.lrn_size <= 0 || d.lrn_size > ly.inC + 64) rc = CG_EINVAL;
            break;
        case CG_LAYER_MAXPOOL:
            if (d.k <= 0 || d.stride <= 0 || d.pad < 0 || d.pad >= d.k) { rc = CG_EINVAL; break; }
            ly.C = ly.inC;
            ly.H = pool_out_size(ly.inH, d.k, d.stride, d.pad);
            ly.W = pool_out_size(ly.inW, d.k, d.stride, d.pad);
            if (ly.H <= 0 || ly.W <= 0) rc = CG_EINVAL;
            ly.aux_elems = (size_t)B * ly.C * ly.H * ly.W;      // argmax (int32)
            break;
        case CG_LAYER_AVGPOOL:
            ly.C = ly.inC; ly.H = ly.W = 1;
            break;
        case CG_LAYER_CONCAT: {
            int cs = 0;
            for (int k = 0; k < d.n_inputs; ++k) {
                int c, h, w;
                in_shape(*net, d.inputs[k], &c, &h, &w);
                if (h != ly.inH || w != ly.inW) rc = CG_EINVAL;
                cs += c;
            }
            ly.C = cs; ly.H = ly.inH; ly.W = ly.inW;
            break;
        }
        case CG_LAYER_SOFTMAX_CE:
            if (i != L - 1 || d.inputs[0] < 0) { rc = CG_EINVAL; break; }
            ly.C = ly.H = ly.W = 1;
            break;
        default:
            rc = CG_EINVAL;
        }
        if (rc) break;
        ly.out_elems = (size_t)B * ly.C * ly.H * ly.W;
        if (ly.out_elems >= (1ull << 29)) { rc = CG_EUNSUPPORTED; break; }
        if (d.kind == CG_LAYER_RELU && d.inputs[0] >= 0) {
            Layer &src = net->layers[d.inputs[0]];
            int consumers = 0;
            for (int j = 0; j < L; ++j)
                for (int k = 0; k < descs[j].n_inputs && k < 4; ++k)
                    if (descs[j].inputs[k] == d.inputs[0]) ++consumers;
            if ((src.d.kind == CG_LAYER_CONV || src.d.kind == CG_LAYER_FC) && consumers == 1) {
                src.fused_relu = true;
                ly.alias_of = d.inputs[0];
            }
        }
        if (ly.alias_of >= 0) ly.act_off = net->layers[ly.alias_of].act_off;
        else { ly.act_off = off; off += round_up(ly.out_elems, 64); }
        ly.grad_off = off; off += round_up(ly.out_elems, 64);
        ly.aux_off = off; off += round_up(ly.aux_elems, 64);
    }
    if (rc == CG_OK) {
        for (int r = 0; r < L; ++r) {
            Layer &rl = net->layers[r];
            if (rl.d.kind != CG_LAYER_RELU || rl.d.inputs[0] < 0 || !net->layers[rl.d.inputs[0]].needs_grad) continue;
            int consumers = 0, who = -1;
            for (int j = r + 1; j < L; ++j)
                for (int k = 0; k < net->layers[j].d.n_inputs; ++k)
                    if (net->layers[j].d.inputs[k] == r) { ++consumers; who = j; }
            if (consumers != 1) continue;
            const int kind = net->layers[who].d.kind;
            const bool can = kind == CG_LAYER_CONV || kind == CG_LAYER_FC || kind == CG_LAYER_LRN ||
                             kind == CG_LAYER_MAXPOOL || kind == CG_LAYER_DROPOUT;
            if (!can) continue;
            rl.bwd_folded = true;
            net->layers[who].gate_from = r;
        }
    }
    if (rc == CG_OK) {
        for (int j = 0; j < L; ++j) {
            Layer &cat = net->layers[j];
            if (cat.d.kind != CG_LAYER_CONCAT) continue;
            int c_off = 0;
            for (int k = 0; k < cat.d.n_inputs; ++k) {
                const int r = cat.d.inputs[k];
                int c, h, w;
                in_shape(*net, r, &c, &h, &w);
                const int my_off = c_off;
                c_off += c;
                if (r < 0) continue;
                Layer &rl = net->layers[r];
                if (rl.d.kind != CG_LAYER_RELU || rl.alias_of < 0 || net->layers[rl.alias_of].d.kind != CG_LAYER_CONV) continue;
                int consumers = 0;
                for (int j2 = 0; j2 < L; ++j2)
                    for (int k2 = 0; k2 < net->layers[j2].d.n_inputs; ++k2)
                        if (net->layers[j2].d.inputs[k2] == r) ++consumers;
                // the slice must start on a 16-byte boundary like every tensor the kernels are given
                if (consumers != 1 || cat.out_elems >= (1ull << 31) || ((size_t)my_off * cat.H * cat.W) % 4 != 0) continue;
                Layer &cv = net->layers[rl.alias_of];
                cv.out_img_stride = rl.out_img_stride = (long long)cat.C * cat.H * cat.W;
                cv.act_off = rl.act_off = cat.act_off + (size_t)my_off * cat.H * cat.W;
                cv.in_concat = rl.in_concat = j;
                if (cv.needs_grad) rl.bwd_folded = true;
            }
        }
    }
    if (rc == CG_OK && g_fuse_lrn_pool.load(std::memory_order_relaxed)) {
        for (int r = 0; r < L; ++r) {
            Layer &ln = net->layers[r];
            if (ln.d.kind != CG_LAYER_LRN) continue;
            int consumers = 0, who = -1;
            for (int j = r + 1; j < L; ++j)
                for (int k = 0; k < net->layers[j].d.n_inputs; ++k)
                    if (net->layers[j].d.inputs[k] == r) { ++consumers; who = j; }
            if (consumers != 1 || net->layers[who].d.kind != CG_LAYER_MAXPOOL) continue;
            const cg_layer_desc &pd = net->layers[who].d;
            if (!lrn_pool_fusable(ln.C, ln.H, ln.W, ln.d.lrn_size, pd.k, pd.stride, pd.pad)) continue;
            ln.fused_pool = who;
            ln.fused_pool_bwd = (g_fuse_lrn_pool.load(std::memory_order_relaxed) & 2) != 0;
            net->layers[who].fused_lrn = r;
        }
    }
    if (rc == CG_OK && net->layers[L - 1].d.kind != CG_LAYER_SOFTMAX_CE) rc = CG_EINVAL;
    if (rc == CG_OK) {
        // the logits feed the loss only: its gradient is written by the loss kernel
        const int src = net->layers[L - 1].d.inputs[0];
        for (int i = 0; i < L - 1; ++i)
            for (int k = 0; k < net->layers[i].d.n_inputs; ++k)
                if (net->layers[i].d.inputs[k] == src) rc = CG_EUNSUPPORTED;
    }
    if (rc == CG_OK) {
        net->loss_off = off; off += round_up((size_t)B, 64);
        for (Layer &ly : net->layers)
            if (ly.d.kind == CG_LAYER_CONV) {
                const size_t n = round_up(conv_filter_prep_max_floats(ly.conv), 64);
                ly.prep_fwd_off = off; off += n;
                ly.prep_bd_off = off; off += n;
            }
        net->scratch_off = off; net->scratch_bytes = round_up(scratch, 256);
        off += 2 * (net->scratch_bytes / sizeof(float));
        net->ws_floats = off;
        for (Layer &ly : net->layers)
            if (ly.n_params) {
                if (hipEventCreateWithFlags(&ly.ev_grad, hipEventDisableTiming) != hipSuccess ||
                    hipEventCreateWithFlags(&ly.ev_upd, hipEventDisableTiming) != hipSuccess ||
                    hipEventCreateWithFlags(&ly.ev_dy, hipEventDisableTiming) != hipSuccess ||
                    hipEventCreateWithFlags(&ly.ev_bd, hipEventDisableTiming) != hipSuccess) { rc = CG_EHIP; break; }
            }
        if (rc == CG_OK && hipStreamCreateWithFlags(&net->wgrad_stream, hipStreamNonBlocking) != hipSuccess) rc = CG_EHIP;
        if (rc == CG_OK && hipEventCreateWithFlags(&net->ev_join, hipEventDisableTiming) != hipSuccess) rc = CG_EHIP;
    }
    if (rc != CG_OK) { cg_net_destroy(net); return rc; }
    *out = net;
    return CG_OK;
}

extern "C" int cg_net_destroy(cg_net *net)
{
    if (!net) return CG_OK;
    for (Layer &ly : net->layers) {
        if (ly.ev_grad) (void)hipEventDestroy(ly.ev_grad);
        if (ly.ev_upd) (void)hipEventDestroy(ly.ev_upd);
        if (ly.ev_dy) (void)hipEventDestroy(ly.ev_dy);
        if (ly.ev_bd) (void)hipEventDestroy(ly.ev_bd);
    }
    if (net->wgrad_stream) (void)hipStreamDestroy(net->wgrad_stream);
    if (net->ev_join) (void)hipEventDestroy(net->ev_join);
    delete net;
    return CG_OK;
}

extern "C" long long cg_net_param_count(const cg_net *net, int layer)
{
    if (!net || layer < 0 || layer >= (int)net->layers.size()) return CG_EINVAL;
    return net->layers[layer].n_params;
}

extern "C" int cg_net_layer_fused(const cg_net *net, int layer)
{
    if (!net || layer < 0 || layer >= (int)net->layers.size()) return CG_EINVAL;
    const cg_net::Layer &ly = net->layers[layer];
    return ((ly.fused_relu || ly.fused_pool >= 0) ? 1 : 0) | ((ly.bwd_folded || ly.fused_pool_bwd) ? 2 : 0);
}

extern "C" int cg_net_bind(cg_net *net, int layer, float *w, float *v, float *g_local, const float *const *g_peers,
                           int K)
{
    if (!net || layer < 0 || layer >= (int)net->layers.size()) return CG_EINVAL;
    Layer &ly = net->layers[layer];
    if (!ly.n_params || !w || !v || !g_local || K < 0 || K > CG_MAX_PEERS || (K > 0 && !g_peers)) return CG_EINVAL;
    if (!aligned16(w) || !aligned16(v) || !aligned16(g_local)) return CG_EINVAL;
    for (int k = 0; k < K; ++k)
        if (!g_peers[k] || !aligned16(g_peers[k])) return CG_EINVAL;
    ly.w = w; ly.v = v; ly.g = g_local;
    ly.peers.assign(g_peers, g_peers + K);
    ly.bound = true;
    return CG_OK;
}

extern "C" size_t cg_net_workspace_bytes(const cg_net *net)
{
    return net ? net->ws_floats * sizeof(float) : 0;
}

extern "C" int cg_net_tensor(const cg_net *net, int layer, int which, void *ws, float **ptr, size_t *count)
{
    if (!net || !ws || !ptr || !count || layer < 0 || layer >= (int)net->layers.size()) return CG_EINVAL;
    const Layer &ly = net->layers[layer];
    float *base = static_cast<float *>(ws);
    if (which == 0) *ptr = base + ly.act_off;
    else if (which == 1) *ptr = base + ly.grad_off;
    else if (which == 2) *ptr = base + ly.aux_off;
    else return CG_EINVAL;
    *count = which == 2 ? ly.aux_elems : ly.out_elems;
    if (which == 0 && ly.out_img_stride)
        *count = (size_t)(net->B - 1) * (size_t)ly.out_img_stride + (size_t)ly.C * ly.H * ly.W;
    return CG_OK;
}

extern "C" long long cg_net_tensor_image_stride(const cg_net *net, int layer)
{
    if (!net || layer < 0 || layer >= (int)net->layers.size()) return CG_EINVAL;
    const Layer &ly = net->layers[layer];
    return ly.out_img_stride ? ly.out_img_stride : (long long)ly.C * ly.H * ly.W;
}

extern "C" int cg_train_step(cg_net *net, const float *x, const int32_t *labels, const uint8_t *const *masks,
                             const cg_sgd *sgd, void *ws, size_t ws_bytes, void *compute_stream,
                             void *update_stream, float *loss_dev, int flags)
{
    if (!net || !x || !labels || !sgd || !ws || !loss_dev) return CG_EINVAL;
    if (ws_bytes < net->ws_floats * sizeof(float)) return CG_ENOSPC;
    if (!aligned16(ws) || !aligned16(x)) return CG_EINVAL;
    const bool serial = (flags & CG_STEP_SERIAL) != 0;
    if ((flags & CG_STEP_BF16) && (flags & CG_STEP_BF16X3)) return CG_EINVAL;
    const int math = (flags & CG_STEP_BF16) ? CG_MATH_BF16 : (flags & CG_STEP_BF16X3) ? CG_MATH_BF16X3 : CG_MATH_FP32;
    hipStream_t S0 = static_cast<hipStream_t>(compute_stream);
    hipStream_t S1 = serial ? S0 : static_cast<hipStream_t>(update_stream);
    if (!serial && S0 == S1) return CG_EINVAL;
    const int L = (int)net->layers.size();
    for (int i = 0; i < L; ++i) {
        const Layer &ly = net->layers[i];
        if (ly.n_params && !ly.bound) return CG_EINVAL;
        if (ly.d.kind == CG_LAYER_DROPOUT && (!masks || !masks[i])) return CG_EINVAL;
    }
    float *base = static_cast<float *>(ws);
    void *scratch = base + net->scratch_off;
    const size_t scratch_bytes = net->scratch_bytes;
    void *scratch2 = serial ? scratch : static_cast<char *>(scratch) + scratch_bytes;
    // Backward-weight of a layer needs only that layer's dy and input, backward-data only dy and the
    // model: the two run side by side, backward-weight on a stream of the net's own, so that the blocks
    // of one fill the compute units the other's last wave of blocks leaves idle.
    hipStream_t S2 = serial ? S0 : net->wgrad_stream;
    hipEvent_t last_wgrad = nullptr;
    const int B = net->B;
    auto act = [&](int i) -> const float * { return i < 0 ? x : base + net->layers[i].act_off; };
    int rc = CG_OK;

    hipEvent_t waited_upd = nullptr;             // the update event the compute stream waited for last

    // ---- the rearranged filter copies of every convolution, for forward and backward-data of this
    // iteration, eight layers a launch (the model changes again only in this iteration's updates).
    // Their layers' updates of the previous call must have landed: the first layer's is the last one
    // the update stream runs, so nothing is lost by waiting for them up front.
    {
        std::vector<FilterPrep> jobs;
        std::vector<const float *> jw;
        std::vector<float *> jd;
        for (int i = 0; i < L; ++i) {
            Layer &ly = net->layers[i];
            if (ly.d.kind != CG_LAYER_CONV) continue;
            ly.prep_fwd = ly.prep_bd = nullptr;
            const FilterPrep f = conv_fwd_filter_prep(ly.conv);
            if (f.kind != CG_PREP_NONE) {
                ly.prep_fwd = base + ly.prep_fwd_off;
                jobs.push_back(f); jw.push_back(ly.w); jd.push_back(base + ly.prep_fwd_off);
            }
            const int s0 = ly.d.inputs[0];
            if (ly.needs_grad && s0 >= 0 && net->layers[s0].needs_grad) {
                const FilterPrep b = conv_bwd_data_filter_prep(ly.conv);
                if (b.kind != CG_PREP_NONE) {
                    ly.prep_bd = base + ly.prep_bd_off;
                    jobs.push_back(b); jw.push_back(ly.w); jd.push_back(base + ly.prep_bd_off);
                }
            }
            if ((ly.prep_fwd || ly.prep_bd) && ly.n_params && ly.upd_pending) {
                if (ly.upd_event != waited_upd) CG_HIP_TRY(hipStreamWaitEvent(S0, ly.upd_event, 0));
                waited_upd = ly.upd_event;
                ly.upd_pending = false;
            }
        }
        if (!jobs.empty()) {
            ProfTag tag("filter_prep", -1);
            rc = filter_prep_launch((int)jobs.size(), jobs.data(), jw.data(), jd.data(), S0);
            if (rc) return rc;
        }
    }

    // ---- forward, layers 1..L --------------------------------------------------------------
    for (int i = 0; i < L && rc == CG_OK; ++i) {
        Layer &ly = net->layers[i];
        const cg_layer_desc &d = ly.d;
        const float *in = act(d.inputs[0]);
        float *out = base + ly.act_off;
        ly.grad_written = false;
        ProfTag tag("", i);
        if (ly.n_params && ly.upd_pending) {
            // finalize, per layer: the model of this layer must have received its update
            if (ly.upd_event != waited_upd) CG_HIP_TRY(hipStreamWaitEvent(S0, ly.upd_event, 0));
            waited_upd = ly.upd_event;
            ly.upd_pending = false;
        }
        const size_t in_elems = (size_t)B * ly.inC * ly.inH * ly.inW;
        switch (d.kind) {
        case CG_LAYER_CONV:
            rc = conv_fwd_impl(ly.conv, in, ly.w, ly.w + ly.n_weights, out, scratch, scratch_bytes, ly.fused_relu, S0,
                               ly.out_img_stride, math, ly.prep_fwd);
            break;
        case CG_LAYER_FC:
            rc = fc_fwd_impl(B, ly.inC * ly.inH * ly.inW, d.fc_out, in, ly.w, ly.w + ly.n_weights, out, scratch,
                             scratch_bytes, ly.fused_relu, S0, math);
            break;
        case CG_LAYER_RELU:
            if (ly.alias_of < 0) rc = relu_fwd_launch(in, out, in_elems, S0);
            break;
        case CG_LAYER_LRN:
            if (ly.fused_pool >= 0) break;           // runs at the pool's place, fused with it
            rc = lrn_fwd_launch(in, out, B, ly.C, ly.H * ly.W, d.lrn_size, d.lrn_alpha, d.lrn_beta, d.lrn_kappa, S0);
            break;
        case CG_LAYER_MAXPOOL:
            if (ly.fused_lrn >= 0) {
                const Layer &ln = net->layers[ly.fused_lrn];
                rc = lrn_pool_fwd_launch(act(ln.d.inputs[0]), out, reinterpret_cast<int32_t *>(base + ly.aux_off), B, ln.C,
                                         ln.H, ln.W, ln.d.lrn_size, ln.d.lrn_alpha, ln.d.lrn_beta, ln.d.lrn_kappa, d.k,
                                         d.stride, d.pad, S0);
                break;
            }
            rc = maxpool_fwd_launch(in, out, reinterpret_cast<int32_t *>(base + ly.aux_off), B, ly.inC, ly.inH,
                                    ly.inW, d.k, d.stride, d.pad, S0);
            break;
        case CG_LAYER_AVGPOOL: rc = avgpool_fwd_launch(in, out, B * ly.inC, ly.inH * ly.inW, S0); break;
        case CG_LAYER_DROPOUT: rc = dropout_launch(in, masks[i], out, nullptr, in_elems, d.drop_p, 0, S0); break;
        case CG_LAYER_CONCAT: {
            int c_off = 0;
            for (int k = 0; k < d.n_inputs && rc == CG_OK; ++k) {
                int c, h, w;
                in_shape(*net, d.inputs[k], &c, &h, &w);
                const bool in_place = d.inputs[k] >= 0 && net->layers[d.inputs[k]].in_concat == i;
                if (!in_place) rc = concat_copy_launch(act(d.inputs[k]), out, B, c, ly.C, c_off, ly.H * ly.W, 1, 0, nullptr, S0);
                c_off += c;
            }
            break;
        }
        case CG_LAYER_SOFTMAX_CE: {
            Layer &src = net->layers[d.inputs[0]];
            rc = softmax_ce_launch(in, labels, loss_dev, base + src.grad_off, base + net->loss_off, B,
                                   src.C * src.H * src.W, S0);
            src.grad_written = true;
            break;
        }
        }
    }
    if (rc) return rc;

    // Layers whose gradients are complete (in stream order) and whose updates have not been launched yet.
    std::vector<int> pend;
    size_t pend_params = 0;
    constexpr long long kBatchParams = 1ll << 20;
    auto flush_updates = [&]() -> int {
        if (pend.empty()) return CG_OK;
        Layer &last = net->layers[pend.back()];
        if (!serial) {
            // the update overwrites the models backward-data reads and consumes the gradients
            // backward-weight writes: it waits for both streams, which run the layers in turn order
            CG_HIP_TRY(hipEventRecord(last.ev_grad, S2));
            CG_HIP_TRY(hipEventRecord(last.ev_bd, S0));
            CG_HIP_TRY(hipStreamWaitEvent(S1, last.ev_grad, 0));
            CG_HIP_TRY(hipStreamWaitEvent(S1, last.ev_bd, 0));
            last_wgrad = last.ev_grad;
        }
        float *w[8], *v[8];
        const float *g[8];
        const float *const *peers[8];
        size_t n[8];
        const int nb = (int)pend.size();
        for (int k = 0; k < nb; ++k) {
            Layer &l = net->layers[pend[k]];
            w[k] = l.w; v[k] = l.v; g[k] = l.g; peers[k] = l.peers.data(); n[k] = (size_t)l.n_params;
        }
        const int rcu = grad_reduce_sgd_multi_impl(nb, w, v, g, peers, (int)last.peers.size(), n, *sgd, S1,
                                                   (flags & CG_STEP_TREE_SUM) != 0);
        if (rcu) return rcu;
        if (!serial) {
            CG_HIP_TRY(hipEventRecord(last.ev_upd, S1));
            for (int k = 0; k < nb; ++k) {
                net->layers[pend[k]].upd_event = last.ev_upd;
                net->layers[pend[k]].upd_pending = true;
            }
        }
        pend.clear();
        pend_params = 0;
        return CG_OK;
    };

    // the layer whose gradient concat layer `cat` writes for its input `sk`: the input itself, or,
    // where the input is a rectifier folded into this concat, the rectifier's producer
    auto concat_target = [&](int cat, int sk) -> int {
        const Layer &src = net->layers[sk];
        return src.bwd_folded && src.in_concat == cat ? src.d.inputs[0] : sk;
    };

    // ---- backward, layers L..1, one turn per layer ----------------------------------------
    for (int i = L - 2; i >= 0 && rc == CG_OK; --i) {
        Layer &ly = net->layers[i];
        const cg_layer_desc &d = ly.d;
        if (!ly.needs_grad) continue;                // no parameter upstream of or inside this layer
        if (ly.bwd_folded) continue;                 // its consumer has already written the gradient of its input
        if (!ly.grad_written) return CG_EINVAL;      // an output nobody consumed
        ProfTag tag("", i);
        const float *dy = base + ly.grad_off;
        const float *in = act(d.inputs[0]);
        const int s0 = d.inputs[0];
        // gradient with respect to the (first) input, if anything upstream needs it; through a folded
        // rectifier the target is the gradient of the rectifier's input, gated by its output
        const bool want_dx = s0 >= 0 && net->layers[s0].needs_grad;
        const int tgt = want_dx && ly.gate_from >= 0 ? net->layers[s0].d.inputs[0] : s0;
        const float *gate = want_dx && ly.gate_from >= 0 ? act(s0) : nullptr;
        float *dx = want_dx ? base + net->layers[tgt].grad_off : nullptr;
        const int accum = want_dx && net->layers[tgt].grad_written ? 1 : 0;
        const size_t in_elems = (size_t)B * ly.inC * ly.inH * ly.inW;
        switch (d.kind) {
        case CG_LAYER_CONV:
        case CG_LAYER_FC: {
            if (!serial) {
                CG_HIP_TRY(hipEventRecord(ly.ev_dy, S0));
                CG_HIP_TRY(hipStreamWaitEvent(S2, ly.ev_dy, 0));
            }
            const int IN = ly.inC * ly.inH * ly.inW;
            if (d.kind == CG_LAYER_CONV)
                // without a backward-data pass of its own (a first layer) the compute stream is idle during this
                // turn: the bias sums go there, beside the weight gradient; the update waits for both streams
                // (their partial sums in the compute stream's own scratch region: the other region may still be
                // read by an earlier layer's weight-gradient kernels, which only the third stream orders)
                rc = conv_bwd_weight_impl(ly.conv, in, dy, ly.g, ly.g + ly.n_weights, scratch2, scratch_bytes, S2, math,
                                          (!serial && !want_dx) ? S0 : nullptr, scratch, scratch_bytes);
            else
                rc = fc_bwd_weight_impl(B, IN, d.fc_out, in, dy, ly.g, ly.g + ly.n_weights, scratch2, scratch_bytes, S2, math);
            if (rc == CG_OK && want_dx) {
                if (d.kind == CG_LAYER_CONV)
                    // (true: the tile choice made for the three-stream schedule, in the one-stream schedule as well,
                    // which thereby issues exactly the same launches, one at a time)
                    rc = conv_bwd_data_impl(ly.conv, dy, ly.w, dx, gate, scratch, scratch_bytes, accum, S0, math, ly.prep_bd,
                                            true);
                else
                    rc = fc_bwd_data_impl(B, IN, d.fc_out, dy, ly.w, dx, gate, accum, scratch, scratch_bytes, S0, math);
            }
            break;
        }
        case CG_LAYER_RELU:
            if (want_dx) rc = relu_bwd_launch(in, dy, dx, in_elems, accum, S0);
            break;
        case CG_LAYER_LRN:
            if (want_dx && ly.fused_pool_bwd) {
                const Layer &pl = net->layers[ly.fused_pool];
                rc = lrn_pool_bwd_launch(in, base + pl.grad_off, reinterpret_cast<const int32_t *>(base + pl.aux_off), dx, B,
                                         ly.C, ly.H, ly.W, d.lrn_size, d.lrn_alpha, d.lrn_beta, d.lrn_kappa, pl.d.k,
                                         pl.d.stride, pl.d.pad, accum, gate != nullptr, S0);
            } else if (want_dx)
                rc = lrn_bwd_launch(in, dy, dx, B, ly.C, ly.H * ly.W, d.lrn_size, d.lrn_alpha, d.lrn_beta,
                                    d.lrn_kappa, accum, gate != nullptr, S0);
            break;
        case CG_LAYER_MAXPOOL:
            if (ly.fused_lrn >= 0 && net->layers[ly.fused_lrn].fused_pool_bwd)
                break;                                   // the LRN's turn goes from this layer's gradient to its own input's
            if (want_dx)
                rc = maxpool_bwd_launch(dy, reinterpret_cast<const int32_t *>(base + ly.aux_off), dx, gate, B, ly.inC,
                                        ly.inH, ly.inW, d.k, d.stride, d.pad, accum, S0);
            break;
        case CG_LAYER_AVGPOOL:
            if (want_dx) rc = avgpool_bwd_launch(dy, dx, B * ly.inC, ly.inH * ly.inW, accum, S0);
            break;
        case CG_LAYER_DROPOUT:
            if (want_dx) rc = dropout_launch(dy, masks[i], dx, gate, in_elems, d.drop_p, accum, S0);
            break;
        case CG_LAYER_CONCAT: {
            int c_off = 0;
            for (int k = 0; k < d.n_inputs && rc == CG_OK; ++k) {
                int c, h, w;
                in_shape(*net, d.inputs[k], &c, &h, &w);
                const int sk = d.inputs[k];
                if (sk >= 0 && net->layers[sk].needs_grad) {
                    const int t = concat_target(i, sk);
                    Layer &T = net->layers[t];
                    // through a folded rectifier: gated by the rectifier's output, which is this
                    // layer's own output slice
                    rc = concat_copy_launch(dy, base + T.grad_off, B, c, ly.C, c_off, ly.H * ly.W, 0,
                                            T.grad_written ? 1 : 0, t != sk ? base + ly.act_off : nullptr, S0);
                    T.grad_written = true;
                }
                c_off += c;
            }
            break;
        }
        default: break;
        }
        if (rc) return rc;
        if (want_dx && d.kind != CG_LAYER_CONCAT) net->layers[tgt].grad_written = true;

        if (ly.n_params) {
            // the turn's second half: aggregate this layer's gradient over the ranks and update its model.
            // Small layers wait for their neighbours: up to eight of them, or a million parameters, go out
            // in one launch (a net of many small layers is bound by the number of launches, and the
            // layer-wise update does not care how many layers a launch carries); a large layer goes at once.
            const bool big = ly.n_params >= kBatchParams;
            if (!pend.empty() && (big || net->layers[pend[0]].peers.size() != ly.peers.size())) {
                rc = flush_updates();
                if (rc) return rc;
            }
            pend.push_back(i);
            pend_params += (size_t)ly.n_params;
            if (big || pend.size() == 8 || pend_params >= (size_t)kBatchParams) rc = flush_updates();
            if (rc) return rc;
        }
    }
    if (rc == CG_OK) rc = flush_updates();
    if (rc) return rc;
    // the local gradients are promised in compute-stream order, and the next call's forward may
    // overwrite what the last backward-weight still reads
    if (!serial && last_wgrad) CG_HIP_TRY(hipStreamWaitEvent(S0, last_wgrad, 0));
    if (rc == CG_OK && !serial && (flags & CG_STEP_JOIN)) {
        // the update stream joins the compute stream as well: nothing of this step is left on a stream
        // the caller has not passed, and the next call waits for no event of this one
        bool any = false;
        for (Layer &ly : net->layers) {
            any = any || ly.upd_pending;
            ly.upd_pending = false;
        }
        if (any) {
            CG_HIP_TRY(hipEventRecord(net->ev_join, S1));
            CG_HIP_TRY(hipStreamWaitEvent(S0, net->ev_join, 0));
        }
    }
    return rc;
}
