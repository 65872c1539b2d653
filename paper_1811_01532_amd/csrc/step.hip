// One replica's whole training step as a precomputed host-side launch list: forward, loss,
// backward, SGD (what each per-GPU partial graph of Section 3.1 executes between two gradient
// aggregations; its duration is the sum over layers of t_c in Eq. 1).  The plan owns no device
// memory: every tensor lives at a fixed offset of one caller-provided arena, all launches go to
// one stream, nothing allocates or synchronises in wap_step_run.
#include <algorithm>
#include <cstring>
#include <string>
#include <utility>
#include <vector>

#include "wap_internal.h"

using namespace wap;

namespace {

enum OpKind {
    OP_PACK, OP_CONV_FWD, OP_POOL_FWD, OP_FC_FWD, OP_SOFTMAX, OP_RELU_BWD, OP_POOL_BWD,
    OP_FC_DX, OP_FC_DW, OP_CONV_WGRAD, OP_CONV_DGRAD, OP_SGD, OP_BIAS_GRAD, OP_BIAS_FINISH
};

struct Tensor {
    std::string name;
    size_t off, bytes;
};

struct Op {
    OpKind kind;
    std::string name;
    GemmGeom gg;
    GemmPlan gp;
    WgradGeom wg;
    WgradPlan wp;
    bool b_tr = false, relu = false;
    bool has_mask = false;  // data gradient fused with the ReLU derivative of the layer below (mask tensor at t3)
    bool prepacked = false;  // weights of this operation are repacked once per step by the OP_PACK operation (copy at t4)
    size_t t0 = 0, t1 = 0, t2 = 0, t3 = 0, t4 = 0, t5 = 0;  // arena offsets, meaning per kind
    bool has_pool = false;  // conv forward whose epilogue also emits the 2x2 max-pool (y_pool at t3, argmax at t5)
    bool has_bias = false;  // forward operation with an fp32 bias vector (at tb)
    size_t tb = 0;
    bool unpool = false;    // conv backward whose dy operand is the gradient of the 2x2-pooled output, routed through the
                            // argmax by the kernel's loader (argmax at t5 for the data gradient, t3 for the weight gradient)
    bool fuse_sgd = false;  // weight gradient that applies the SGD update itself (fp32 master weights at t6, bf16 copy at
                            // t7); it runs after the layer's data gradient, which still needs the old weights
    size_t t6 = 0, t7 = 0;
    bool colsum = false;    // data gradient whose epilogue also leaves per-tile column sums of its (masked) output at t8:
                            // the bias gradient of the layer below, finished by the OP_BIAS_FINISH operation behind it
    size_t t8 = 0;
    int N = 0, H = 0, W = 0, C = 0, win = 0, st = 0;  // pooling / softmax shapes
    size_t n = 0;
    const char* kernel = "";  // kernel instantiation the operation launches
    double flops = 0, bytes = 0;  // algorithmic work: operands read once, outputs written once
};

struct ConvL {
    const char* name;
    int C, K, R, stride, pad, pool_win, pool_st;
};
struct FcL {
    const char* name;
    int out;
    bool relu;
};

const ConvL kAlexConvs[] = {
    {"conv1", 3, 64, 11, 4, 2, 3, 2}, {"conv2", 64, 192, 5, 1, 2, 3, 2}, {"conv3", 192, 384, 3, 1, 1, 0, 0},
    {"conv4", 384, 256, 3, 1, 1, 0, 0}, {"conv5", 256, 256, 3, 1, 1, 3, 2},
};
const ConvL kVggConvs[] = {
    {"conv1_1", 3, 64, 3, 1, 1, 0, 0},    {"conv1_2", 64, 64, 3, 1, 1, 2, 2},   {"conv2_1", 64, 128, 3, 1, 1, 0, 0},
    {"conv2_2", 128, 128, 3, 1, 1, 2, 2}, {"conv3_1", 128, 256, 3, 1, 1, 0, 0}, {"conv3_2", 256, 256, 3, 1, 1, 0, 0},
    {"conv3_3", 256, 256, 3, 1, 1, 2, 2}, {"conv4_1", 256, 512, 3, 1, 1, 0, 0}, {"conv4_2", 512, 512, 3, 1, 1, 0, 0},
    {"conv4_3", 512, 512, 3, 1, 1, 2, 2}, {"conv5_1", 512, 512, 3, 1, 1, 0, 0}, {"conv5_2", 512, 512, 3, 1, 1, 0, 0},
    {"conv5_3", 512, 512, 3, 1, 1, 2, 2},
};
const FcL kFcs[] = {{"fc6", 4096, true}, {"fc7", 4096, true}, {"fc8", 1000, false}};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

struct wap_step_plan {
    std::vector<Tensor> tensors;
    std::vector<Op> ops;
    size_t arena = 0;
    double flops = 0;
    float lr = 0.01f;
    int B = 0, classes = 1000;
    size_t ws_off = 0, ws_bytes = 0;
    size_t n_params = 0;
    size_t w32_off = 0, dw_off = 0, wb_off = 0;
    mutable std::vector<hipEvent_t> events;  // cached by wap_step_time
    PackJobs packjobs = {};                  // every weight repacking of the step, run as one kernel
    ColsumJobs colsumjobs = {};              // every bias gradient finished from per-tile column sums, run as one pair
    mutable bool ran_once = false;           // an eager step has completed its launches (kernel attributes are set)
    hipGraph_t graph = nullptr;
    hipGraphExec_t graph_exec = nullptr;
    void* graph_arena = nullptr;

    size_t add(const std::string& name, size_t bytes) {
        size_t off = arena;
        tensors.push_back({name, off, bytes});
        arena = align_up(arena + bytes, 256);
        return off;
    }
    size_t find(const std::string& name) const {
        for (const Tensor& t : tensors)
            if (t.name == name) return t.off;
        return (size_t)-1;
    }
};

namespace {

int run_op(const wap_step_plan* p, const Op& op, unsigned char* base, hipStream_t st, hipEvent_t ev_mid = nullptr,
           hipEvent_t ev_packed = nullptr) {
    void* ws = base + p->ws_off;
    switch (op.kind) {
        case OP_PACK:
            return launch_pack_weights_multi(p->packjobs, base, st);
        case OP_CONV_FWD:
        case OP_FC_FWD:
        case OP_CONV_DGRAD:
        case OP_FC_DX:
            return launch_fwd_like(op.gg, op.b_tr, op.gp, (const bf16_t*)(base + op.t0), (const bf16_t*)(base + op.t1),
                                   op.has_bias ? (const float*)(base + op.tb) : nullptr, op.relu, op.has_pool ? nullptr : (bf16_t*)(base + op.t2), ws, st, ev_mid,
                                   op.has_mask ? (const bf16_t*)(base + op.t3) : nullptr, ev_packed,
                                   op.prepacked ? (const void*)(base + op.t4) : nullptr,
                                   op.has_pool ? (bf16_t*)(base + op.t3) : nullptr,
                                   op.has_pool ? (uint8_t*)(base + op.t5) : nullptr,
                                   op.unpool ? (const uint8_t*)(base + op.t5) : nullptr,
                                   op.colsum ? (float*)(base + op.t8) : nullptr);
        case OP_CONV_WGRAD:
        case OP_FC_DW: {
            const SgdFuse sgd = {(float*)(base + op.t6), (bf16_t*)(base + op.t7), p->lr};
            return launch_wgrad(op.wg, op.wp, (const bf16_t*)(base + op.t0), (const bf16_t*)(base + op.t1),
                                (float*)(base + op.t2), ws, st, ev_mid,
                                op.unpool ? (const uint8_t*)(base + op.t3) : nullptr, op.fuse_sgd ? &sgd : nullptr);
        }
        case OP_POOL_FWD:
            return launch_maxpool_fwd(op.N, op.H, op.W, op.C, op.win, op.st, (const bf16_t*)(base + op.t0),
                                      (bf16_t*)(base + op.t1), (uint8_t*)(base + op.t2), st);
        case OP_POOL_BWD:
            return launch_maxpool_bwd(op.N, op.H, op.W, op.C, op.win, op.st, (const bf16_t*)(base + op.t0),
                                      (const uint8_t*)(base + op.t1), (const bf16_t*)(base + op.t2),
                                      (bf16_t*)(base + op.t3), st);
        case OP_RELU_BWD:
            return launch_relu_bwd((const bf16_t*)(base + op.t0), (const bf16_t*)(base + op.t1),
                                   (bf16_t*)(base + op.t2), op.n, st);
        case OP_SOFTMAX:
            return launch_softmax_xent(op.N, op.C, (const bf16_t*)(base + op.t0), (const int32_t*)(base + op.t1),
                                       (float*)(base + op.t2), (float*)(base + op.t3), (bf16_t*)(base + op.t4), st);
        case OP_BIAS_GRAD:
            return launch_bias_grad(op.n, op.C, (const bf16_t*)(base + op.t0), (float*)(base + op.t1), (float*)ws, st);
        case OP_BIAS_FINISH:  // the per-tile column sums that the data gradients left -> bias gradients, all layers at once
            return launch_colsum_f32_multi(p->colsumjobs, base, st);
        case OP_SGD:
            return launch_sgd(op.n, (float*)(base + op.t0), (const float*)(base + op.t1), p->lr,
                              (bf16_t*)(base + op.t2), st);
    }
    return set_error(WAP_EINVAL, "internal: unknown op");
}

}  // namespace

extern "C" {

int wap_step_plan_create(const char* net, int32_t minibatch, int32_t image, float lr, uint32_t flags,
                         wap_step_plan** out) {
    if (!net || !out) return set_error(WAP_EINVAL, "step plan: NULL argument");
    if (minibatch < 1 || image < 1) return set_error(WAP_EINVAL, "step plan: minibatch and image must be >= 1");
    if (flags & ~7u) return set_error(WAP_EINVAL, "step plan: unknown flag bits 0x%x", flags);
    const ConvL* convs;
    int nconv;
    if (!strcmp(net, "alexnet")) { convs = kAlexConvs; nconv = 5; }
    else if (!strcmp(net, "vgg16")) { convs = kVggConvs; nconv = 13; }
    else return set_error(WAP_EINVAL, "step plan: unknown net '%s' (alexnet, vgg16)", net);
    const bool keep = (flags & WAP_STEP_KEEP_GRADS) != 0;
    const bool with_bias = (flags & WAP_STEP_BIAS) != 0;
    const bool fuse_update = !keep && (flags & WAP_STEP_STORE_GRADS) == 0;
    const int B = minibatch;

    // ---- walk the geometry, validating every layer ----
    std::vector<wap_conv_desc> cds(nconv);
    std::vector<int> out_hw(nconv), out_ch(nconv);
    int h = image;
    for (int i = 0; i < nconv; ++i) {
        const ConvL& L = convs[i];
        wap_conv_desc d = {B, h, h, L.C, L.K, L.R, L.R, L.stride, L.stride, L.pad, L.pad, WAP_RELU};
        int rc = validate_conv(&d);
        if (rc != WAP_OK) return rc;
        cds[i] = d;
        h = (h + 2 * L.pad - L.R) / L.stride + 1;
        if (L.pool_win) {
            if (h < L.pool_win) return set_error(WAP_EINVAL, "step plan: image %d too small for %s's pool", image, L.name);
            h = (h - L.pool_win) / L.pool_st + 1;
        }
        out_hw[i] = h;
        out_ch[i] = L.K;
    }
    const int flat = h * h * convs[nconv - 1].K;
    std::vector<wap_fc_desc> fds(3);
    int in_f = flat;
    for (int i = 0; i < 3; ++i) {
        wap_fc_desc d = {B, in_f, kFcs[i].out, kFcs[i].relu ? WAP_RELU : 0u};
        int rc = validate_fc(&d);
        if (rc != WAP_OK) return rc;
        fds[i] = d;
        in_f = kFcs[i].out;
    }

    wap_step_plan* p = new wap_step_plan();
    p->B = B;
    p->lr = lr;

    // ---- parameters: three parallel blocks in the same layer order (one SGD launch) ----
    std::vector<size_t> poff(nconv + 3), pcount(nconv + 3);
    size_t np = 0;
    for (int i = 0; i < nconv + 3; ++i) {
        size_t cnt = i < nconv ? (size_t)convs[i].K * convs[i].R * convs[i].R * convs[i].C
                               : (size_t)fds[i - nconv].out_features * fds[i - nconv].in_features;
        poff[i] = np;
        pcount[i] = cnt;
        np += align_up(cnt, 64);
    }
    // biases (optional) follow the weights in the same three blocks, so the one SGD launch covers them
    std::vector<size_t> boff(nconv + 3, 0), bcount(nconv + 3, 0);
    if (with_bias)
        for (int i = 0; i < nconv + 3; ++i) {
            boff[i] = np;
            bcount[i] = i < nconv ? (size_t)convs[i].K : (size_t)fds[i - nconv].out_features;
            np += align_up(bcount[i], 64);
        }
    p->n_params = np;
    p->w32_off = p->add("params.w32", np * 4);
    p->dw_off = p->add("params.dw", np * 4);
    p->wb_off = p->add("params.w", np * 2);
    auto lname = [&](int i) { return std::string(i < nconv ? convs[i].name : kFcs[i - nconv].name); };
    for (int i = 0; i < nconv + 3; ++i) {
        p->tensors.push_back({lname(i) + ".w32", p->w32_off + poff[i] * 4, pcount[i] * 4});
        p->tensors.push_back({lname(i) + ".dw", p->dw_off + poff[i] * 4, pcount[i] * 4});
        p->tensors.push_back({lname(i) + ".w", p->wb_off + poff[i] * 2, pcount[i] * 2});
        if (with_bias) {
            p->tensors.push_back({lname(i) + ".b32", p->w32_off + boff[i] * 4, bcount[i] * 4});
            p->tensors.push_back({lname(i) + ".db", p->dw_off + boff[i] * 4, bcount[i] * 4});
        }
    }

    // ---- activations ----
    size_t t_input = p->add("input", (size_t)B * image * image * 3 * 2);
    size_t t_labels = p->add("labels", (size_t)B * 4);
    size_t t_loss = p->add("loss", 16);
    size_t t_rowloss = p->add("row_loss", (size_t)B * 4);
    std::vector<size_t> conv_y(nconv), pool_y(nconv, 0), pool_am(nconv, 0), conv_y_elems(nconv), pool_y_elems(nconv, 0);
    size_t max_g_elems = (size_t)B * 1000;
    for (int i = 0; i < nconv; ++i) {
        const wap_conv_desc& d = cds[i];
        int P = (d.H + 2 * d.pad_h - d.R) / d.stride_h + 1;
        conv_y_elems[i] = (size_t)B * P * P * d.K;
        conv_y[i] = p->add(lname(i) + ".y", conv_y_elems[i] * 2);
        if (conv_y_elems[i] > max_g_elems) max_g_elems = conv_y_elems[i];
        if (convs[i].pool_win) {
            pool_y_elems[i] = (size_t)B * out_hw[i] * out_hw[i] * d.K;
            pool_y[i] = p->add(lname(i) + ".pool.y", pool_y_elems[i] * 2);
            pool_am[i] = p->add(lname(i) + ".pool.argmax", pool_y_elems[i]);
        }
    }
    std::vector<size_t> fc_y(3);
    for (int i = 0; i < 3; ++i) {
        fc_y[i] = p->add(lname(nconv + i) + ".y", (size_t)B * fds[i].out_features * 2);
        if ((size_t)B * fds[i].in_features > max_g_elems) max_g_elems = (size_t)B * fds[i].in_features;
    }
    size_t gbuf[2] = {0, 0};
    if (!keep) {
        gbuf[0] = p->add("gradbuf0", max_g_elems * 2);
        gbuf[1] = p->add("gradbuf1", max_g_elems * 2);
    }
    int gsel = 0;
    auto new_grad = [&](const std::string& name, size_t elems) -> size_t {
        if (keep) return p->add(name, elems * 2);
        size_t off = gbuf[gsel];
        gsel ^= 1;
        return off;
    };

    size_t ws_need = 0;
    auto push_fwd_like = [&](OpKind kind, const std::string& name, const GemmGeom& g, bool b_tr, bool relu, size_t a,
                             size_t w, size_t o) {
        Op op;
        op.kind = kind; op.name = name; op.gg = g; op.b_tr = b_tr; op.relu = relu;
        op.gp = plan_fwd_like(g, b_tr);
        op.kernel = fwd_like_kernel_name(g, b_tr, op.gp);
        op.flops = 2.0 * g.M * (double)g.Ncols * g.Kred;
        op.bytes = 2.0 * ((double)B * g.IH * g.IW * g.IC + (double)g.Kred * g.Ncols + (double)g.M * g.Ncols);
        op.t0 = a; op.t1 = w; op.t2 = o;
        if (op.gp.ws_bytes > ws_need) ws_need = op.gp.ws_bytes;
        // kernels that read the weights in MFMA fragment order: one repacking kernel per step serves them all
        if ((op.gp.cfg == 6 || op.gp.cfg == 7) && p->packjobs.n < kMaxPackJobs) {
            op.prepacked = true;
            op.t4 = p->add("wpack." + name, wreg_wt_bytes(g));
            pack_jobs_add(p->packjobs, g, b_tr, w, op.t4);
        }
        p->ops.push_back(op);
    };
    // gradient of layer `li`'s bias: column sums of the gradient w.r.t. its pre-activation output (rows x cols, bf16)
    auto push_bias_grad = [&](int li, size_t rows, size_t dy) {
        if (!with_bias) return;
        Op op;
        op.kind = OP_BIAS_GRAD; op.name = lname(li) + ".bias_grad";
        op.n = rows; op.C = (int)bcount[li];
        op.t0 = dy; op.t1 = p->dw_off + boff[li] * 4;
        op.kernel = "bias_grad_kernel";
        op.bytes = 2.0 * rows * bcount[li] + 4.0 * bcount[li];
        size_t need = (size_t)bias_grad_chunks(rows, op.C) * op.C * sizeof(float);
        if (need > ws_need) ws_need = need;
        p->ops.push_back(op);
    };
    // The same gradient where the data gradient that produced dy (ReLU derivative applied in its epilogue) can leave
    // per-tile column sums of what it stores: no pass over dy at all; the (small) partial rows of all such layers are
    // added up by one operation at the end of the backward pass.
    struct ColsumReq { size_t op_index; int li, rows, cols; };
    std::vector<ColsumReq> colsum_reqs;
    auto try_fuse_bias_grad = [&](int li) -> bool {
        if (!with_bias || keep || p->ops.empty() || (int)colsum_reqs.size() >= kMaxColsumJobs) return false;
        Op& prod = p->ops.back();
        if ((prod.kind != OP_CONV_DGRAD && prod.kind != OP_FC_DX) || !prod.has_mask || prod.has_pool) return false;
        const int rows = fwd_like_colsum_rows(prod.gg, prod.gp);
        if (rows == 0 || prod.gg.Ncols != (int)bcount[li] || (prod.gg.Ncols % 4) != 0) return false;
        prod.colsum = true;
        prod.name += "+bias_grad";
        prod.bytes += 4.0 * rows * prod.gg.Ncols;
        colsum_reqs.push_back({p->ops.size() - 1, li, rows, prod.gg.Ncols});
        return true;
    };
    auto set_bias = [&](int li) {
        if (!with_bias) return;
        Op& f = p->ops.back();
        f.has_bias = true;
        f.tb = p->w32_off + boff[li] * 4;
    };
    // Parameter ranges [first, last) whose update is applied by the kernel that finishes the layer's weight gradient:
    // the gradient is then neither stored nor read back.  The kept-gradients layout stores every gradient instead.
    std::vector<std::pair<size_t, size_t>> fused_ranges;
    auto push_wgrad = [&](OpKind kind, const std::string& name, const WgradGeom& g, size_t x, size_t dy, int li) {
        Op op;
        op.kind = kind; op.name = name; op.wg = g;
        op.wp = plan_wgrad(g);
        op.kernel = wgrad_kernel_name(g, op.wp);
        const double nw = (double)g.K * g.R * g.S * g.C;
        op.flops = 2.0 * g.N * g.P * g.Q * nw;
        op.bytes = 2.0 * ((double)g.N * g.H * g.W * g.C + (double)g.N * g.P * g.Q * g.K) + 4.0 * nw;
        op.t0 = x; op.t1 = dy; op.t2 = p->dw_off + poff[li] * 4;
        if (fuse_update && (poff[li] & 3) == 0 && wgrad_fuses_sgd(g, op.wp)) {
            op.fuse_sgd = true;
            op.t6 = p->w32_off + poff[li] * 4;
            op.t7 = p->wb_off + poff[li] * 2;
            op.name += "+sgd";
            op.bytes += 6.0 * nw;  // master weights read and written, bf16 copy written, gradient not stored
            fused_ranges.push_back({poff[li], poff[li] + (size_t)nw});
        }
        if (op.wp.ws_bytes > ws_need) ws_need = op.wp.ws_bytes;
        p->ops.push_back(op);
    };

    // ---- forward ----
    double flops = 0;
    size_t cur = t_input;
    for (int i = 0; i < nconv; ++i) {
        const wap_conv_desc& d = cds[i];
        GemmGeom g = geom_conv_fwd(d);
        push_fwd_like(OP_CONV_FWD, lname(i) + ".fwd", g, false, true, cur, p->wb_off + poff[i] * 2, conv_y[i]);
        set_bias(i);
        double f = 2.0 * g.M * (double)g.Ncols * g.Kred;
        flops += (i == 0 ? 2.0 : 3.0) * f;
        cur = conv_y[i];
        // conv -> ReLU -> 2x2 pool: where the conv kernel can pool in its own epilogue the full-size output is never
        // written (the backward pass needs only the pooled activations and the argmax); the kept-gradients layout
        // keeps the two operations apart for inspection
        if (convs[i].pool_win == 2 && convs[i].pool_st == 2 && !keep && fwd_like_fuses_pool(g, p->ops.back().gp)) {
            Op& cf = p->ops.back();
            cf.has_pool = true;
            cf.t3 = pool_y[i];
            cf.t5 = pool_am[i];
            cf.name = lname(i) + ".fwd+pool";
            cf.bytes += 3.0 * pool_y_elems[i] - 2.0 * conv_y_elems[i];
            cur = pool_y[i];
        } else if (convs[i].pool_win) {
            Op op;
            op.kind = OP_POOL_FWD; op.name = lname(i) + ".pool.fwd";
            op.N = B; op.H = g.OH; op.W = g.OW; op.C = d.K; op.win = convs[i].pool_win; op.st = convs[i].pool_st;
            op.t0 = cur; op.t1 = pool_y[i]; op.t2 = pool_am[i];
            op.kernel = "maxpool_fwd_kernel";
            op.bytes = 2.0 * conv_y_elems[i] + 3.0 * pool_y_elems[i];
            p->ops.push_back(op);
            cur = pool_y[i];
        }
    }
    std::vector<size_t> fc_in(3);
    for (int i = 0; i < 3; ++i) {
        fc_in[i] = cur;
        GemmGeom g = geom_fc_fwd(fds[i]);
        push_fwd_like(OP_FC_FWD, lname(nconv + i) + ".fwd", g, false, kFcs[i].relu, cur, p->wb_off + poff[nconv + i] * 2,
                      fc_y[i]);
        set_bias(nconv + i);
        flops += 3.0 * 2.0 * B * (double)fds[i].in_features * fds[i].out_features;
        cur = fc_y[i];
    }
    p->flops = flops;

    // ---- loss ----
    size_t g_cur = new_grad("g.fc8.y", (size_t)B * 1000);
    {
        Op op;
        op.kind = OP_SOFTMAX; op.name = "softmax_xent";
        op.N = B; op.C = 1000;
        op.t0 = fc_y[2]; op.t1 = t_labels; op.t2 = t_loss; op.t3 = t_rowloss; op.t4 = g_cur;
        op.kernel = "softmax_xent_kernel";
        op.bytes = 4.0 * B * 1000;
        p->ops.push_back(op);
    }

    // ---- backward: FC head ----
    for (int i = 2; i >= 0; --i) {
        std::string nm = lname(nconv + i);
        size_t elems = (size_t)B * fds[i].out_features;
        if (kFcs[i].relu) {
            Op op;
            op.kind = OP_RELU_BWD; op.name = nm + ".relu_bwd";
            op.n = elems;
            op.t0 = g_cur; op.t1 = fc_y[i];
            op.t2 = keep ? p->add("gm." + nm + ".y", elems * 2) : g_cur;
            op.kernel = "relu_bwd_kernel";
            op.bytes = 6.0 * elems;
            p->ops.push_back(op);
            g_cur = op.t2;
        }
        push_wgrad(OP_FC_DW, nm + ".dW", geom_fc_dw(fds[i]), fc_in[i], g_cur, nconv + i);
        push_bias_grad(nconv + i, (size_t)B, g_cur);
        if (!keep) gsel = (g_cur == gbuf[0]) ? 1 : 0;
        std::string in_name = i > 0 ? "g." + lname(nconv + i - 1) + ".y"
                                    : "g." + lname(nconv - 1) + (convs[nconv - 1].pool_win ? ".pool.y" : ".y");
        size_t g_in = new_grad(in_name, (size_t)B * fds[i].in_features);
        push_fwd_like(OP_FC_DX, nm + ".dx", geom_fc_dx(fds[i]), true, false, g_cur, p->wb_off + poff[nconv + i] * 2, g_in);
        g_cur = g_in;
    }

    // ---- backward: conv stack ----
    bool relu_done = false;  // the gradient in g_cur already carries this layer's ReLU derivative
    for (int i = nconv - 1; i >= 0; --i) {
        std::string nm = lname(i);
        const wap_conv_desc& d = cds[i];
        GemmGeom gf = geom_conv_fwd(d);
        if (!keep) gsel = (g_cur == gbuf[0]) ? 1 : 0;
        // conv -> ReLU -> 2x2 pool, backward: where both backward kernels of this layer can route the pooled gradient
        // through the argmax in their own loaders, the full-size gradient is never written.  The ReLU derivative then
        // rides on the producer of the pooled gradient (the routed value is the window's maximum, so the pooled
        // activation decides it).  The kept-gradients layout keeps the steps apart for inspection.
        bool unpool = false;
        if (!keep && convs[i].pool_win == 2 && convs[i].pool_st == 2 && (gf.OH % 2) == 0 && (gf.OW % 2) == 0) {
            const WgradGeom wgm = geom_conv_wgrad(d);
            const GemmGeom dgm = geom_conv_dgrad(d);
            unpool = wgrad_fuses_unpool(wgm, plan_wgrad(wgm)) &&
                     (i == 0 || fwd_like_fuses_unpool(dgm, plan_fwd_like(dgm, true)));
        }
        if (unpool) {
            Op& prod = p->ops.back();  // the data gradient of the layer above (conv or fc6): it wrote g_cur
            prod.has_mask = true;
            prod.t3 = pool_y[i];
            prod.name += "+relu_bwd";
            prod.bytes += 2.0 * pool_y_elems[i];
        } else if (convs[i].pool_win) {
            Op op;
            op.kind = OP_POOL_BWD; op.name = nm + ".pool_relu_bwd";
            op.N = B; op.H = gf.OH; op.W = gf.OW; op.C = d.K; op.win = convs[i].pool_win; op.st = convs[i].pool_st;
            op.t0 = g_cur; op.t1 = pool_am[i]; op.t2 = pool_y[i];
            op.t3 = new_grad("gm." + nm + ".y", conv_y_elems[i]);
            op.kernel = "maxpool_bwd_kernel";
            op.bytes = 2.0 * conv_y_elems[i] + 5.0 * pool_y_elems[i];
            p->ops.push_back(op);
            g_cur = op.t3;
        } else if (!relu_done) {
            Op op;
            op.kind = OP_RELU_BWD; op.name = nm + ".relu_bwd";
            op.n = conv_y_elems[i];
            op.t0 = g_cur; op.t1 = conv_y[i];
            op.t2 = keep ? p->add("gm." + nm + ".y", conv_y_elems[i] * 2) : g_cur;
            op.kernel = "relu_bwd_kernel";
            op.bytes = 6.0 * conv_y_elems[i];
            p->ops.push_back(op);
            g_cur = op.t2;
        }
        // bias gradient: from the epilogue of the data gradient that produced g_cur where that kernel can (it applied
        // this layer's ReLU derivative and is the last operation so far), else a pass over g_cur further down
        const bool bias_fused = (unpool || relu_done) && try_fuse_bias_grad(i);
        size_t x_in = i == 0 ? t_input : (convs[i - 1].pool_win ? pool_y[i - 1] : conv_y[i - 1]);
        push_wgrad(OP_CONV_WGRAD, nm + ".wgrad", geom_conv_wgrad(d), x_in, g_cur, i);
        if (unpool) {
            Op& wgop = p->ops.back();
            wgop.unpool = true;
            wgop.t3 = pool_am[i];
            wgop.name = nm + (wgop.fuse_sgd ? ".unpool+wgrad+sgd" : ".unpool+wgrad");
            wgop.kernel = wgrad_kernel_name(wgop.wg, wgop.wp, true);
            wgop.bytes += 3.0 * pool_y_elems[i] - 2.0 * conv_y_elems[i];
        }
        // routing a pooled gradient to the argmax pixels keeps every column's sum: the pooled tensor serves as well
        if (!bias_fused) push_bias_grad(i, (unpool ? pool_y_elems[i] : conv_y_elems[i]) / d.K, g_cur);
        if (i > 0) {  // the gradient w.r.t. the input image is not needed
            if (!keep) gsel = (g_cur == gbuf[0]) ? 1 : 0;
            std::string in_name = "g." + lname(i - 1) + (convs[i - 1].pool_win ? ".pool.y" : ".y");
            size_t g_in = new_grad(in_name, (size_t)B * d.H * d.W * d.C);
            push_fwd_like(OP_CONV_DGRAD, nm + ".dgrad", geom_conv_dgrad(d), true, false, g_cur, p->wb_off + poff[i] * 2,
                          g_in);
            // When the layer below feeds this one directly (no pool in between) its ReLU derivative is applied in
            // this data gradient's epilogue; the kept-gradients layout keeps the two steps apart for inspection.
            relu_done = false;
            Op& dg = p->ops.back();
            if (unpool) {
                dg.unpool = true;
                dg.t5 = pool_am[i];
                dg.name = nm + ".unpool+dgrad";
                dg.kernel = fwd_like_kernel_name(dg.gg, true, dg.gp, true);
                dg.bytes += 3.0 * pool_y_elems[i] - 2.0 * conv_y_elems[i];
            }
            if (!keep && !convs[i - 1].pool_win && fwd_like_fuses_mask(dg.gg, dg.gp)) {
                dg.has_mask = true;
                dg.t3 = conv_y[i - 1];
                dg.name += "+relu_bwd";
                dg.bytes += 2.0 * conv_y_elems[i - 1];
                relu_done = true;
            }
            g_cur = g_in;
        }
    }

    // ---- bias gradients left as per-tile column sums by the data gradients: one region per layer, finished together ----
    if (!colsum_reqs.empty()) {
        double bytes = 0;
        for (const ColsumReq& rq : colsum_reqs) {
            const size_t part = p->add("bias.colsum." + lname(rq.li), (size_t)rq.rows * rq.cols * sizeof(float));
            const size_t part2 = p->add("bias.colsum2." + lname(rq.li),
                                        (size_t)colsum_f32_chunks((size_t)rq.rows) * rq.cols * sizeof(float));
            p->ops[rq.op_index].t8 = part;
            colsum_jobs_add(p->colsumjobs, rq.rows, rq.cols, part, part2, p->dw_off + boff[rq.li] * 4);
            bytes += 4.0 * rq.rows * rq.cols + 4.0 * rq.cols;
        }
        Op op;
        op.kind = OP_BIAS_FINISH; op.name = "bias_grad_finish";
        op.kernel = "colsum_f32_multi_kernel";
        op.bytes = bytes;
        p->ops.push_back(op);
    }

    // ---- update ----
    // A weight gradient that applies its own update moves behind its layer's data gradient (the next data-gradient
    // operation in the list), which reads the weights of this step; nothing in between touches its operands.
    // (Walking the list from its end, a moved operation lands behind the cursor and is not met again.)
    for (size_t i = p->ops.size(); i-- > 0;) {
        if (!p->ops[i].fuse_sgd) continue;
        size_t j = i + 1;
        while (j < p->ops.size() && p->ops[j].kind != OP_FC_DX && p->ops[j].kind != OP_CONV_DGRAD) ++j;
        if (j == p->ops.size()) continue;  // first layer: no data gradient
        std::rotate(p->ops.begin() + i, p->ops.begin() + i + 1, p->ops.begin() + j + 1);
    }
    // the remaining parameters (gradients stored by their kernels, biases) are updated by one pass per gap
    {
        std::sort(fused_ranges.begin(), fused_ranges.end());
        fused_ranges.push_back({np, np});
        size_t pos = 0;
        int gaps = 0;
        for (const auto& fr : fused_ranges) {
            if (fr.first > pos) {
                Op op;
                op.kind = OP_SGD; op.name = gaps == 0 ? "sgd" : "sgd." + std::to_string(gaps);
                op.n = fr.first - pos;
                op.t0 = p->w32_off + pos * 4; op.t1 = p->dw_off + pos * 4; op.t2 = p->wb_off + pos * 2;
                op.kernel = "sgd_kernel";
                op.bytes = 14.0 * op.n;
                p->ops.push_back(op);
                ++gaps;
            }
            if (fr.second > pos) pos = fr.second;
        }
    }
    if (p->packjobs.n > 0) {
        Op op;
        op.kind = OP_PACK; op.name = "pack_weights";
        op.kernel = "pack_weights_multi_kernel";
        op.bytes = 2.0 * 16.0 * (double)p->packjobs.first[p->packjobs.n];
        p->ops.insert(p->ops.begin(), op);
    }
    p->ws_bytes = ws_need;
    p->ws_off = p->add("workspace", ws_need ? ws_need : 256);
    *out = p;
    return WAP_OK;
}

void wap_step_plan_destroy(wap_step_plan* p) {
    if (!p) return;
    for (hipEvent_t e : p->events) (void)hipEventDestroy(e);
    if (p->graph_exec) (void)hipGraphExecDestroy(p->graph_exec);
    if (p->graph) (void)hipGraphDestroy(p->graph);
    delete p;
}

int wap_step_arena_bytes(const wap_step_plan* p, size_t* bytes_out) {
    if (!p || !bytes_out) return set_error(WAP_EINVAL, "step: NULL argument");
    *bytes_out = p->arena;
    return WAP_OK;
}

int wap_step_num_tensors(const wap_step_plan* p) { return p ? (int)p->tensors.size() : 0; }

int wap_step_tensor(const wap_step_plan* p, int32_t index, const char** name, size_t* offset, size_t* bytes) {
    if (!p || !name || !offset || !bytes) return set_error(WAP_EINVAL, "step: NULL argument");
    if (index < 0 || index >= (int)p->tensors.size()) return set_error(WAP_EINVAL, "step: tensor index %d out of range", index);
    *name = p->tensors[index].name.c_str();
    *offset = p->tensors[index].off;
    *bytes = p->tensors[index].bytes;
    return WAP_OK;
}

double wap_step_flops(const wap_step_plan* p) { return p ? p->flops : 0.0; }
int wap_step_num_ops(const wap_step_plan* p) { return p ? (int)p->ops.size() : 0; }

static int check_arena(const wap_step_plan* p, void* arena, size_t arena_bytes) {
    if (!p || !arena) return set_error(WAP_EINVAL, "step: NULL argument");
    if ((reinterpret_cast<uintptr_t>(arena) & 255u) != 0) return set_error(WAP_EINVAL, "step: arena is not 256-byte aligned");
    if (arena_bytes < p->arena) return set_error(WAP_EWORKSPACE, "step: arena has %zu bytes, %zu needed", arena_bytes, p->arena);
    return WAP_OK;
}

int wap_step_run(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream) {
    int rc = check_arena(p, arena, arena_bytes);
    if (rc != WAP_OK) return rc;
    unsigned char* base = (unsigned char*)arena;
    for (const Op& op : p->ops) {
        rc = run_op(p, op, base, (hipStream_t)stream);
        if (rc != WAP_OK) return rc;
    }
    p->ran_once = true;
    return WAP_OK;
}

int wap_step_graph_capture(wap_step_plan* p, void* arena, size_t arena_bytes, void* stream) {
    int rc = check_arena(p, arena, arena_bytes);
    if (rc != WAP_OK) return rc;
    if (!p->ran_once) return set_error(WAP_EINVAL, "step graph: run one eager step (wap_step_run) before capturing");
    if (!stream) return set_error(WAP_EINVAL, "step graph: capture needs an explicit (non-default) stream");
    hipStream_t st = (hipStream_t)stream;
    if (p->graph_exec) { (void)hipGraphExecDestroy(p->graph_exec); p->graph_exec = nullptr; }
    if (p->graph) { (void)hipGraphDestroy(p->graph); p->graph = nullptr; }
    hipError_t e = hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return set_error(WAP_EHIP, "hipStreamBeginCapture: %s", hipGetErrorString(e));
    unsigned char* base = (unsigned char*)arena;
    for (const Op& op : p->ops) {
        rc = run_op(p, op, base, st);
        if (rc != WAP_OK) break;
    }
    hipGraph_t g = nullptr;
    e = hipStreamEndCapture(st, &g);
    if (rc != WAP_OK) {
        if (g) (void)hipGraphDestroy(g);
        return rc;
    }
    if (e != hipSuccess || !g) return set_error(WAP_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
    hipGraphExec_t ge = nullptr;
    e = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGraphDestroy(g);
        return set_error(WAP_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e));
    }
    p->graph = g;
    p->graph_exec = ge;
    p->graph_arena = arena;
    return WAP_OK;
}

int wap_step_graph_launch(const wap_step_plan* p, void* stream) {
    if (!p) return set_error(WAP_EINVAL, "step graph: NULL plan");
    if (!p->graph_exec) return set_error(WAP_EINVAL, "step graph: nothing captured");
    hipError_t e = hipGraphLaunch(p->graph_exec, (hipStream_t)stream);
    if (e != hipSuccess) return set_error(WAP_EHIP, "hipGraphLaunch: %s", hipGetErrorString(e));
    return WAP_OK;
}

int wap_step_op_info(const wap_step_plan* p, int32_t index, const char** name, const char** kernel,
                     double* flops, double* bytes) {
    if (!p || !name || !kernel || !flops || !bytes) return set_error(WAP_EINVAL, "step: NULL argument");
    if (index < 0 || index >= (int)p->ops.size()) return set_error(WAP_EINVAL, "step: op index %d out of range", index);
    const Op& op = p->ops[index];
    *name = op.name.c_str();
    *kernel = op.kernel;
    *flops = op.flops;
    *bytes = op.bytes;
    return WAP_OK;
}

int wap_step_time(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream, int32_t steps,
                  float* us_out, float* us_epilogue_out) {
    return wap_step_time_masked(p, arena, arena_bytes, stream, steps, nullptr, us_out, us_epilogue_out, nullptr);
}

int wap_step_time_masked(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream, int32_t steps,
                         const uint8_t* op_mask, float* us_out, float* us_epilogue_out, float* us_prologue_out) {
    return wap_step_time_sampled(p, arena, arena_bytes, stream, steps, 1, op_mask, us_out, us_epilogue_out,
                                 us_prologue_out);
}

int wap_step_time_sampled(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream, int32_t steps,
                          int32_t every, const uint8_t* op_mask, float* us_out, float* us_epilogue_out,
                          float* us_prologue_out) {
    int rc = check_arena(p, arena, arena_bytes);
    if (rc != WAP_OK) return rc;
    if (!us_out || !us_epilogue_out || steps < 1 || every < 1) return set_error(WAP_EINVAL, "step: bad argument");
    const int timed = (steps + every - 1) / every;  // steps 0, every, 2 * every, ... carry the events
    unsigned char* base = (unsigned char*)arena;
    hipStream_t st = (hipStream_t)stream;
    const size_t n = p->ops.size();
    const size_t need = 4 * n * (size_t)timed;
    while (p->events.size() < need) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return set_error(WAP_EHIP, "hipEventCreate failed");
        p->events.push_back(e);
    }
    auto has_epilogue = [&](const Op& op) {
        switch (op.kind) {
            case OP_CONV_FWD: case OP_FC_FWD: case OP_CONV_DGRAD: case OP_FC_DX: return op.gp.nsplit > 1;
            case OP_CONV_WGRAD: case OP_FC_DW: return op.wp.nsplit > 1;
            default: return false;
        }
    };
    auto has_prologue = [&](const Op& op) {
        switch (op.kind) {
            case OP_CONV_FWD: case OP_FC_FWD: case OP_CONV_DGRAD: case OP_FC_DX:
                return fwd_like_packs_weights(op.gp) && !op.prepacked;
            default: return false;
        }
    };
    for (int s = 0; s < steps && rc == WAP_OK; ++s)
        for (size_t i = 0; i < n && rc == WAP_OK; ++i) {
            hipEvent_t* ev = &p->events[4 * ((size_t)(s / every) * n + i)];
            if ((s % every) != 0 || (op_mask && !op_mask[i])) {
                rc = run_op(p, p->ops[i], base, st, nullptr);
                continue;
            }
            (void)hipEventRecord(ev[0], st);
            rc = run_op(p, p->ops[i], base, st, has_epilogue(p->ops[i]) ? ev[2] : nullptr,
                        has_prologue(p->ops[i]) ? ev[3] : nullptr);
            (void)hipEventRecord(ev[1], st);
        }
    hipError_t e = hipStreamSynchronize(st);
    if (rc == WAP_OK && e != hipSuccess) rc = set_error(WAP_EHIP, "step: %s", hipGetErrorString(e));
    if (rc != WAP_OK) return rc;
    for (size_t i = 0; i < n; ++i) {
        double sum = 0, sum_epi = 0;
        const bool epi = has_epilogue(p->ops[i]);
        if (us_prologue_out) us_prologue_out[i] = 0.f;
        if (op_mask && !op_mask[i]) {
            us_out[i] = 0.f;
            us_epilogue_out[i] = 0.f;
            continue;
        }
        const bool pro = has_prologue(p->ops[i]);
        double sum_pro = 0;
        for (int s = 0; s < timed; ++s) {
            float ms = 0.f;
            hipEvent_t* ev = &p->events[4 * ((size_t)s * n + i)];
            hipEvent_t first = ev[0];
            if (pro) {
                (void)hipEventElapsedTime(&ms, ev[0], ev[3]);
                sum_pro += ms;
                first = ev[3];
            }
            if (epi) {
                (void)hipEventElapsedTime(&ms, first, ev[2]);
                sum += ms;
                (void)hipEventElapsedTime(&ms, ev[2], ev[1]);
                sum_epi += ms;
            } else {
                (void)hipEventElapsedTime(&ms, first, ev[1]);
                sum += ms;
            }
        }
        if (us_prologue_out) us_prologue_out[i] = (float)(sum_pro * 1000.0 / timed);
        us_out[i] = (float)(sum * 1000.0 / timed);
        us_epilogue_out[i] = (float)(sum_epi * 1000.0 / timed);
    }
    return WAP_OK;
}

}  // extern "C"
