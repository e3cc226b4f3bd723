// The networks of the workloads as fixed launch sequences (internal, see model.hpp), and the
// host-only queries about their parameter vector and workspace.
#include <algorithm>
#include <cstdio>
#include <vector>

#include "../../include/dssp.h"
#include "../../include/dssp_kernels.h"
#include "model.hpp"

namespace dssp_model {

namespace {

struct Seg { int32_t kind; int64_t size, fan_in; };
enum { KW_ = 0, KB_ = 1, KG_ = 2, KBETA_ = 3 };

bool is_resnet(int id) { return id >= 8 && (id - 2) % 6 == 0; }

struct ResBlock {
    int H, cin, cout, stride;              // H: input height = width
    int64_t w1, g1, b1, w2, g2, b2;        // offsets into the flat parameter vector (floats)
    size_t c1, a1, c2, out, st1, st2;      // offsets into the worker's workspace slice (bytes)
};

// Bump allocator over one worker's slice of the workspace (256-byte granules).
struct Arena {
    size_t off = 0;
    size_t take(size_t bytes) { const size_t o = off; off += (bytes + 255) / 256 * 256; return o; }
    size_t floats(size_t n) { return take(n * sizeof(float)); }
};

}  // namespace

struct Plan {
    int model_id = 0, m = 0, n_classes = 0, K = 0;
    char* ws = nullptr;
    size_t per_worker = 0;
    std::vector<Seg> segs;
    int64_t n_params = 0;
    // tensors tests may look at: (what, byte offset in the worker slice, element count)
    struct Tens { int what; size_t off; int64_t count; };
    std::vector<Tens> tens;

    // common tail
    size_t logits = 0, dlogits = 0, fc_scratch = 0, colsum_scratch = 0, wg_scratch = 0, wg_scratch2 = 0, bn_scratch = 0, bn_scratch2 = 0, tot_a = 0, tot_b = 0;
    // MLP
    size_t mlp_a1 = 0, mlp_da1 = 0;
    // AlexNet-style
    size_t ax_a1 = 0, ax_p1 = 0, ax_arg1 = 0, ax_a2 = 0, ax_p2 = 0, ax_arg2 = 0, ax_a3 = 0, ax_a4 = 0;
    size_t ax_da4 = 0, ax_da3 = 0, ax_dp2 = 0, ax_da2 = 0, ax_dp1 = 0, ax_da1 = 0;
    size_t ax_c3 = 0, ax_dc3 = 0;     // three-convolution variant: conv3 output (post-ReLU) and its gradient
    // ResNet
    std::vector<ResBlock> blocks;
    int64_t stem_w = 0, stem_g = 0, stem_b = 0, fc_w = 0, fc_b = 0;
    size_t stem_c = 0, stem_a = 0, stem_st = 0, pooled = 0, dpooled = 0, G[3] = {0, 0, 0};

    void seg(int kind, int64_t size, int64_t fan_in) { segs.push_back({kind, size, fan_in}); n_params += size; }
    int64_t conv_seg(int k, int cin, int cout, bool bias) {
        const int64_t o = n_params;
        seg(KW_, (int64_t)k * k * cin * cout, (int64_t)k * k * cin);
        if (bias) seg(KB_, cout, 0);
        return o;
    }
    int64_t fc_seg(int in, int out) {
        const int64_t o = n_params;
        seg(KW_, (int64_t)in * out, in);
        seg(KB_, out, 0);
        return o;
    }
    int64_t bn_seg(int c) {
        const int64_t o = n_params;
        seg(KG_, c, 0);
        seg(KBETA_, c, 0);
        return o;
    }

    bool build(int id, int batch, int classes) {
        model_id = id; m = batch; n_classes = classes;
        Arena a;
        size_t wg = 0, bn = 0;
        auto wg_need = [&](int N, int H, int Cin, int Cout, int k, int s, int p) {
            const size_t f = dsspk_conv_wgrad_scratch_floats(N, H, H, Cin, Cout, k, k, s, p);
            if (f > wg) wg = f;
        };
        auto bn_need = [&](long M, int C) { const size_t f = dsspk_bn_scratch_floats(M, C); if (f > bn) bn = f; };
        if (id == DSSP_MODEL_MLP) {
            fc_seg(3072, 256);
            fc_seg(256, classes);
            mlp_a1 = a.floats((size_t)m * 256);
            mlp_da1 = a.floats((size_t)m * 256);
            tens.push_back({0, mlp_a1, (int64_t)m * 256});
        } else if (id == DSSP_MODEL_ALEXNET_DS) {
            conv_seg(5, 3, 64, true);
            conv_seg(5, 64, 64, true);
            fc_seg(7 * 7 * 64, 384);
            fc_seg(384, 192);
            fc_seg(192, classes);
            const size_t s32 = (size_t)m * 32 * 32 * 64, s15 = (size_t)m * 15 * 15 * 64, s7 = (size_t)m * 7 * 7 * 64;
            ax_a1 = a.floats(s32); ax_p1 = a.floats(s15); ax_arg1 = a.take(s15);
            ax_a2 = a.floats(s15); ax_p2 = a.floats(s7); ax_arg2 = a.take(s7);
            ax_a3 = a.floats((size_t)m * 384); ax_a4 = a.floats((size_t)m * 192);
            ax_da4 = a.floats((size_t)m * 192); ax_da3 = a.floats((size_t)m * 384); ax_dp2 = a.floats(s7);
            ax_da2 = a.floats(s15); ax_dp1 = a.floats(s15); ax_da1 = a.floats(s32);
            wg_need(m, 32, 3, 64, 5, 1, 2);
            wg_need(m, 15, 64, 64, 5, 1, 2);
            tens.push_back({0, ax_a1, (int64_t)s32}); tens.push_back({0, ax_a2, (int64_t)s15});
            tens.push_back({0, ax_a3, (int64_t)m * 384}); tens.push_back({0, ax_a4, (int64_t)m * 192});
            tens.push_back({1, ax_arg1, (int64_t)s15}); tens.push_back({1, ax_arg2, (int64_t)s7});
        } else if (id == DSSP_MODEL_ALEXNET_3C) {
            conv_seg(5, 3, 64, true);
            conv_seg(5, 64, 64, true);
            conv_seg(3, 64, 64, true);
            fc_seg(7 * 7 * 64, 384);
            fc_seg(384, classes);
            const size_t s32 = (size_t)m * 32 * 32 * 64, s15 = (size_t)m * 15 * 15 * 64, s7 = (size_t)m * 7 * 7 * 64, s7c = s7;
            ax_a1 = a.floats(s32); ax_p1 = a.floats(s15); ax_arg1 = a.take(s15);
            ax_a2 = a.floats(s15); ax_p2 = a.floats(s7); ax_arg2 = a.take(s7);
            ax_c3 = a.floats(s7c); ax_a3 = a.floats((size_t)m * 384);
            ax_da3 = a.floats((size_t)m * 384); ax_dc3 = a.floats(s7c); ax_dp2 = a.floats(s7);
            ax_da2 = a.floats(s15); ax_dp1 = a.floats(s15); ax_da1 = a.floats(s32);
            wg_need(m, 32, 3, 64, 5, 1, 2);
            wg_need(m, 15, 64, 64, 5, 1, 2);
            wg_need(m, 7, 64, 64, 3, 1, 1);
            tens.push_back({0, ax_a1, (int64_t)s32}); tens.push_back({0, ax_a2, (int64_t)s15});
            tens.push_back({0, ax_c3, (int64_t)s7c}); tens.push_back({0, ax_a3, (int64_t)m * 384});
            tens.push_back({1, ax_arg1, (int64_t)s15}); tens.push_back({1, ax_arg2, (int64_t)s7});
        } else if (is_resnet(id)) {
            const int n = (id - 2) / 6;
            stem_w = conv_seg(3, 3, 16, false);
            stem_g = bn_seg(16); stem_b = stem_g + 16;
            const size_t s0 = (size_t)m * 32 * 32 * 16;
            stem_c = a.floats(s0); stem_a = a.floats(s0); stem_st = a.floats(32);
            tens.push_back({0, stem_a, (int64_t)s0});
            wg_need(m, 32, 3, 16, 3, 1, 1);
            bn_need((long)m * 32 * 32, 16);
            int cin = 16, H = 32;
            const int widths[3] = {16, 32, 64};
            for (int st = 0; st < 3; ++st)
                for (int b = 0; b < n; ++b) {
                    ResBlock B;
                    B.cin = cin; B.cout = widths[st]; B.stride = (st > 0 && b == 0) ? 2 : 1; B.H = H;
                    const int Ho = H / B.stride;
                    B.w1 = conv_seg(3, B.cin, B.cout, false); B.g1 = bn_seg(B.cout); B.b1 = B.g1 + B.cout;
                    B.w2 = conv_seg(3, B.cout, B.cout, false); B.g2 = bn_seg(B.cout); B.b2 = B.g2 + B.cout;
                    const size_t sz = (size_t)m * Ho * Ho * B.cout;
                    B.c1 = a.floats(sz); B.a1 = a.floats(sz); B.c2 = a.floats(sz); B.out = a.floats(sz);
                    B.st1 = a.floats(2 * B.cout); B.st2 = a.floats(2 * B.cout);
                    tens.push_back({0, B.a1, (int64_t)sz}); tens.push_back({0, B.out, (int64_t)sz});
                    wg_need(m, H, B.cin, B.cout, 3, B.stride, 1);
                    wg_need(m, Ho, B.cout, B.cout, 3, 1, 1);
                    bn_need((long)m * Ho * Ho, B.cout);
                    blocks.push_back(B);
                    cin = B.cout; H = Ho;
                }
            fc_w = fc_seg(64, classes); fc_b = fc_w + 64 * (int64_t)classes;
            pooled = a.floats((size_t)m * 64); dpooled = a.floats((size_t)m * 64);
            for (int i = 0; i < 3; ++i) G[i] = a.floats(s0);
        } else {
            return false;
        }
        logits = a.floats((size_t)m * classes);
        dlogits = a.floats((size_t)m * classes);
        tens.push_back({2, logits, (int64_t)m * classes});
        // split-K scratch of the wide fully connected forward product (3136 -> 384)
        fc_scratch = a.floats(id == DSSP_MODEL_ALEXNET_DS ? (size_t)dsspk_gemm_splitk_layers(m, 384, 3136) * m * 384
                              : id == DSSP_MODEL_ALEXNET_3C ? (size_t)dsspk_gemm_splitk_layers(m, 384, 3136) * m * 384 : 1);
        {
            size_t cs = 1;
            if (id == DSSP_MODEL_ALEXNET_DS || id == DSSP_MODEL_ALEXNET_3C) cs = dsspk_colsum_scratch_floats((long)m * 32 * 32, 64) + 1;
            colsum_scratch = a.floats(cs);
        }
        wg_scratch = a.floats(wg ? wg : 1);
        wg_scratch2 = a.floats(is_resnet(id) && wg ? wg : 1);   // d-filter partial sums alternate between the two
        bn_scratch = a.floats(bn ? bn : 1);
        bn_scratch2 = a.floats(bn ? bn : 1);
        tot_a = a.floats(128); tot_b = a.floats(128);          // batch-norm backward sums (2 x 64 channels at most)
        per_worker = a.off;
        return true;
    }
};

namespace {

#define RUN(call)                                                        \
    do {                                                                 \
        const int rc_ = (call);                                          \
        if (rc_) { err = #call; return rc_; }                            \
    } while (0)

int step_mlp(Plan* P, char* ws, void* s, const float* x, const int32_t* y, const float* w, float* g, float* loss, std::string& err) {
    const int m = P->m, C = P->n_classes;
    float* a1 = (float*)(ws + P->mlp_a1); float* da1 = (float*)(ws + P->mlp_da1);
    float* z = (float*)(ws + P->logits); float* dz = (float*)(ws + P->dlogits);
    const int64_t w1 = 0, b1 = 3072 * 256, w2 = b1 + 256, b2 = w2 + 256 * (int64_t)C;
    RUN(dsspk_gemm(s, x, 3072, 1, w + w1, 256, 1, a1, 256, m, 256, 3072, w + b1, 1));   // (split-K: one more launch, and this net is bound by launches)
    RUN(dsspk_gemm(s, a1, 256, 1, w + w2, C, 1, z, C, m, C, 256, w + b2, 0));
    RUN(dsspk_softmax_xent(s, z, y, dz, loss, m, C));
    RUN(dsspk_gemm(s, a1, 1, 256, dz, C, 1, g + w2, C, 256, C, m, nullptr, 0));          // dW2 = a1^T dz
    RUN(dsspk_colsum(s, dz, g + b2, nullptr, m, C));
    RUN(dsspk_gemm(s, dz, C, 1, w + w2, 1, C, da1, 256, m, 256, C, nullptr, 0));         // da1 = dz W2^T
    RUN(dsspk_relu_bwd(s, da1, a1, (long)m * 256));
    RUN(dsspk_gemm(s, x, 1, 3072, da1, 256, 1, g + w1, 256, 3072, 256, m, nullptr, 0));  // dW1 = x^T dz1
    RUN(dsspk_colsum(s, da1, g + b1, nullptr, m, 256));
    return 0;
}

int step_alexnet(Plan* P, char* ws, void* s, const float* x, const int32_t* y, const float* w, float* g, float* loss, std::string& err) {
    const int m = P->m, C = P->n_classes;
    auto F = [&](size_t off) { return (float*)(ws + off); };
    float *a1 = F(P->ax_a1), *p1 = F(P->ax_p1), *a2 = F(P->ax_a2), *p2 = F(P->ax_p2), *a3 = F(P->ax_a3), *a4 = F(P->ax_a4);
    uint8_t *arg1 = (uint8_t*)(ws + P->ax_arg1), *arg2 = (uint8_t*)(ws + P->ax_arg2);
    float *z = F(P->logits), *dz = F(P->dlogits), *da4 = F(P->ax_da4), *da3 = F(P->ax_da3), *dp2 = F(P->ax_dp2);
    float *da2 = F(P->ax_da2), *dp1 = F(P->ax_dp1), *da1 = F(P->ax_da1), *scr = F(P->wg_scratch);
    const int64_t cw1 = 0, cb1 = 4800, cw2 = cb1 + 64, cb2 = cw2 + 102400, fw1 = cb2 + 64, fb1 = fw1 + 3136 * 384,
                  fw2 = fb1 + 384, fb2 = fw2 + 384 * 192, fw3 = fb2 + 192, fb3 = fw3 + 192 * (int64_t)C;
    // forward
    RUN(dsspk_conv_fwd(s, x, w + cw1, w + cb1, a1, m, 32, 32, 3, 64, 5, 5, 1, 2, 1, nullptr));
    RUN(dsspk_maxpool_fwd(s, a1, p1, arg1, m, 32, 32, 64));
    RUN(dsspk_conv_fwd(s, p1, w + cw2, w + cb2, a2, m, 15, 15, 64, 64, 5, 5, 1, 2, 1, nullptr));
    RUN(dsspk_maxpool_fwd(s, a2, p2, arg2, m, 15, 15, 64));
    RUN(dsspk_gemm_splitk(s, p2, 3136, 1, w + fw1, 384, 1, a3, 384, m, 384, 3136, w + fb1, 1, F(P->fc_scratch),
                          dsspk_gemm_splitk_layers(m, 384, 3136)));
    RUN(dsspk_gemm(s, a3, 384, 1, w + fw2, 192, 1, a4, 192, m, 192, 384, w + fb2, 1));
    RUN(dsspk_gemm(s, a4, 192, 1, w + fw3, C, 1, z, C, m, C, 192, w + fb3, 0));
    RUN(dsspk_softmax_xent(s, z, y, dz, loss, m, C));
    // backward
    RUN(dsspk_gemm(s, a4, 1, 192, dz, C, 1, g + fw3, C, 192, C, m, nullptr, 0));
    RUN(dsspk_colsum(s, dz, g + fb3, nullptr, m, C));
    RUN(dsspk_gemm(s, dz, C, 1, w + fw3, 1, C, da4, 192, m, 192, C, nullptr, 0));
    RUN(dsspk_relu_bwd(s, da4, a4, (long)m * 192));
    RUN(dsspk_gemm(s, a3, 1, 384, da4, 192, 1, g + fw2, 192, 384, 192, m, nullptr, 0));
    RUN(dsspk_colsum(s, da4, g + fb2, nullptr, m, 192));
    RUN(dsspk_gemm(s, da4, 192, 1, w + fw2, 1, 192, da3, 384, m, 384, 192, nullptr, 0));
    RUN(dsspk_relu_bwd(s, da3, a3, (long)m * 384));
    RUN(dsspk_gemm(s, p2, 1, 3136, da3, 384, 1, g + fw1, 384, 3136, 384, m, nullptr, 0));
    RUN(dsspk_colsum(s, da3, g + fb1, nullptr, m, 384));
    RUN(dsspk_gemm(s, da3, 384, 1, w + fw1, 1, 384, dp2, 3136, m, 3136, 384, nullptr, 0));
    RUN(dsspk_maxpool_bwd_relu(s, dp2, arg2, a2, da2, m, 15, 15, 64));
    RUN(dsspk_conv_bwd_weight(s, p1, da2, g + cw2, scr, m, 15, 15, 64, 64, 5, 5, 1, 2));
    RUN(dsspk_colsum(s, da2, g + cb2, F(P->colsum_scratch), (long)m * 15 * 15, 64));
    RUN(dsspk_conv_bwd_data(s, da2, w + cw2, nullptr, dp1, m, 15, 15, 64, 64, 5, 5, 1, 2));
    RUN(dsspk_maxpool_bwd_relu(s, dp1, arg1, a1, da1, m, 32, 32, 64));
    RUN(dsspk_conv_bwd_weight(s, x, da1, g + cw1, scr, m, 32, 32, 3, 64, 5, 5, 1, 2));
    RUN(dsspk_colsum(s, da1, g + cb1, F(P->colsum_scratch), (long)m * 32 * 32, 64));
    return 0;
}

// The reduced AlexNet with three convolutional and two fully connected layers (Sec. V-A3); the layers and kernels of
// step_alexnet in a different order.
int step_alexnet3(Plan* P, char* ws, void* s, const float* x, const int32_t* y, const float* w, float* g, float* loss, std::string& err) {
    const int m = P->m, C = P->n_classes;
    auto F = [&](size_t off) { return (float*)(ws + off); };
    float *a1 = F(P->ax_a1), *p1 = F(P->ax_p1), *a2 = F(P->ax_a2), *p2 = F(P->ax_p2), *c3 = F(P->ax_c3), *a3 = F(P->ax_a3);
    uint8_t *arg1 = (uint8_t*)(ws + P->ax_arg1), *arg2 = (uint8_t*)(ws + P->ax_arg2);
    float *z = F(P->logits), *dz = F(P->dlogits), *da3 = F(P->ax_da3), *dc3 = F(P->ax_dc3), *dp2 = F(P->ax_dp2);
    float *da2 = F(P->ax_da2), *dp1 = F(P->ax_dp1), *da1 = F(P->ax_da1), *scr = F(P->wg_scratch), *cscr = F(P->colsum_scratch);
    const int64_t cw1 = 0, cb1 = 4800, cw2 = cb1 + 64, cb2 = cw2 + 102400, cw3 = cb2 + 64, cb3 = cw3 + 36864,
                  fw1 = cb3 + 64, fb1 = fw1 + 3136 * 384, fw2 = fb1 + 384, fb2 = fw2 + 384 * (int64_t)C;
    // forward
    RUN(dsspk_conv_fwd(s, x, w + cw1, w + cb1, a1, m, 32, 32, 3, 64, 5, 5, 1, 2, 1, nullptr));
    RUN(dsspk_maxpool_fwd(s, a1, p1, arg1, m, 32, 32, 64));
    RUN(dsspk_conv_fwd(s, p1, w + cw2, w + cb2, a2, m, 15, 15, 64, 64, 5, 5, 1, 2, 1, nullptr));
    RUN(dsspk_maxpool_fwd(s, a2, p2, arg2, m, 15, 15, 64));
    RUN(dsspk_conv_fwd(s, p2, w + cw3, w + cb3, c3, m, 7, 7, 64, 64, 3, 3, 1, 1, 1, nullptr));
    RUN(dsspk_gemm_splitk(s, c3, 3136, 1, w + fw1, 384, 1, a3, 384, m, 384, 3136, w + fb1, 1, F(P->fc_scratch),
                          dsspk_gemm_splitk_layers(m, 384, 3136)));
    RUN(dsspk_gemm(s, a3, 384, 1, w + fw2, C, 1, z, C, m, C, 384, w + fb2, 0));
    RUN(dsspk_softmax_xent(s, z, y, dz, loss, m, C));
    // backward
    RUN(dsspk_gemm(s, a3, 1, 384, dz, C, 1, g + fw2, C, 384, C, m, nullptr, 0));
    RUN(dsspk_colsum(s, dz, g + fb2, nullptr, m, C));
    RUN(dsspk_gemm(s, dz, C, 1, w + fw2, 1, C, da3, 384, m, 384, C, nullptr, 0));
    RUN(dsspk_relu_bwd(s, da3, a3, (long)m * 384));
    RUN(dsspk_gemm(s, c3, 1, 3136, da3, 384, 1, g + fw1, 384, 3136, 384, m, nullptr, 0));
    RUN(dsspk_colsum(s, da3, g + fb1, nullptr, m, 384));
    RUN(dsspk_gemm(s, da3, 384, 1, w + fw1, 1, 384, dc3, 3136, m, 3136, 384, nullptr, 0));
    RUN(dsspk_relu_bwd(s, dc3, c3, (long)m * 3136));
    RUN(dsspk_conv_bwd_weight(s, p2, dc3, g + cw3, scr, m, 7, 7, 64, 64, 3, 3, 1, 1));
    RUN(dsspk_colsum(s, dc3, g + cb3, cscr, (long)m * 7 * 7, 64));
    RUN(dsspk_conv_bwd_data(s, dc3, w + cw3, nullptr, dp2, m, 7, 7, 64, 64, 3, 3, 1, 1));
    RUN(dsspk_maxpool_bwd_relu(s, dp2, arg2, a2, da2, m, 15, 15, 64));
    RUN(dsspk_conv_bwd_weight(s, p1, da2, g + cw2, scr, m, 15, 15, 64, 64, 5, 5, 1, 2));
    RUN(dsspk_colsum(s, da2, g + cb2, cscr, (long)m * 15 * 15, 64));
    RUN(dsspk_conv_bwd_data(s, da2, w + cw2, nullptr, dp1, m, 15, 15, 64, 64, 5, 5, 1, 2));
    RUN(dsspk_maxpool_bwd_relu(s, dp1, arg1, a1, da1, m, 32, 32, 64));
    RUN(dsspk_conv_bwd_weight(s, x, da1, g + cw1, scr, m, 32, 32, 3, 64, 5, 5, 1, 2));
    RUN(dsspk_colsum(s, da1, g + cb1, cscr, (long)m * 32 * 32, 64));
    return 0;
}

int step_resnet(Plan* P, char* ws, void* s, const float* x, const int32_t* y, const float* w, float* g, float* loss, std::string& err) {
    const int m = P->m, C = P->n_classes;
    const float eps = 1e-5f;
    auto F = [&](size_t off) { return (float*)(ws + off); };
    float *scr = F(P->wg_scratch), *bscr = F(P->bn_scratch);
    // ---- forward
    RUN(dsspk_conv_fwd(s, x, w + P->stem_w, nullptr, F(P->stem_c), m, 32, 32, 3, 16, 3, 3, 1, 1, 0, nullptr));
    RUN(dsspk_bn_fwd(s, F(P->stem_c), w + P->stem_g, w + P->stem_b, F(P->stem_a), F(P->stem_st), bscr,
                     (long)m * 1024, 16, eps, 1, 0, nullptr, 0, 0, 0, 0));
    // Statistics records ping-pong between two buffers: conv1 writes recA, conv2 reads recA and writes recB,
    // the next block's conv1 reads recB.  A "regular" block (stride 1, same width, shape covered by the specialised
    // kernels) has its two batch norms folded into the loaders of the convolutions that consume them:
    //   conv1 [+ BN2/shortcut/ReLU of the previous block in its loader]  ->  conv2 [+ BN1/ReLU in its loader]
    // and only the last block of a run materialises its output with the stand-alone BN kernels.
    float *recA = bscr, *recB = F(P->bn_scratch2);
    const int nb = (int)P->blocks.size();
    auto regular = [&](int i) {
        const ResBlock& b = P->blocks[i];
        return b.stride == 1 && b.cin == b.cout && dsspk_conv_fwd_stat_parts(m, b.H, b.H, b.cin, b.cout, 3, 3, 1, 1) > 0;
    };
    const float* cur = F(P->stem_a);
    bool pending = false;            // the previous block's output is not written yet (its BN2 is folded into this conv1)
    for (int bi = 0; bi < nb; ++bi) {
        const ResBlock& B = P->blocks[bi];
        const int Ho = B.H / B.stride;
        const long M = (long)m * Ho * Ho;
        const int parts1 = dsspk_conv_fwd_stat_parts(m, B.H, B.H, B.cin, B.cout, 3, 3, B.stride, 1);
        const int parts2 = dsspk_conv_fwd_stat_parts(m, Ho, Ho, B.cout, B.cout, 3, 3, 1, 1);
        if (pending) {
            const ResBlock& Pv = P->blocks[bi - 1];
            const float* pin = bi >= 2 ? F(P->blocks[bi - 2].out) : F(P->stem_a);         // the previous block's input = its shortcut
            RUN(dsspk_conv_fwd_prebn(s, F(Pv.c2), recB, parts2, w + Pv.g2, w + Pv.b2, eps, pin, F(Pv.out), F(Pv.st2),
                                     w + B.w1, F(B.c1), recA, m, B.H, B.cin));
        } else {
            RUN(dsspk_conv_fwd(s, cur, w + B.w1, nullptr, F(B.c1), m, B.H, B.H, B.cin, B.cout, 3, 3, B.stride, 1, 0, parts1 ? recA : nullptr));
        }
        if (parts1 && parts2) {
            RUN(dsspk_conv_fwd_prebn(s, F(B.c1), recA, parts1, w + B.g1, w + B.b1, eps, nullptr, F(B.a1), F(B.st1),
                                     w + B.w2, F(B.c2), recB, m, Ho, B.cout));
        } else {
            RUN(dsspk_bn_fwd(s, F(B.c1), w + B.g1, w + B.b1, F(B.a1), F(B.st1), recA, M, B.cout, eps, 1, 0, nullptr, 0, 0, 0, parts1));
            RUN(dsspk_conv_fwd(s, F(B.a1), w + B.w2, nullptr, F(B.c2), m, Ho, Ho, B.cout, B.cout, 3, 3, 1, 1, 0, parts2 ? recB : nullptr));
        }
        pending = regular(bi) && parts2 > 0 && bi + 1 < nb && regular(bi + 1);
        if (!pending) {
            const int mode = (B.stride == 1 && B.cin == B.cout) ? 1 : 2;
            RUN(dsspk_bn_fwd(s, F(B.c2), w + B.g2, w + B.b2, F(B.out), F(B.st2), recB, M, B.cout, eps, 1, mode, cur, m, Ho, Ho, parts2));
        }
        cur = F(B.out);
    }
    RUN(dsspk_gap_fwd(s, cur, F(P->pooled), m, 64, 64));
    RUN(dsspk_gemm(s, F(P->pooled), 64, 1, w + P->fc_w, C, 1, F(P->logits), C, m, C, 64, w + P->fc_b, 0));
    RUN(dsspk_softmax_xent(s, F(P->logits), y, F(P->dlogits), loss, m, C));
    // ---- backward
    RUN(dsspk_gemm(s, F(P->pooled), 1, 64, F(P->dlogits), C, 1, g + P->fc_w, C, 64, C, m, nullptr, 0));
    RUN(dsspk_colsum(s, F(P->dlogits), g + P->fc_b, nullptr, m, C));
    RUN(dsspk_gemm(s, F(P->dlogits), C, 1, w + P->fc_w, 1, C, F(P->dpooled), 64, m, 64, C, nullptr, 0));
    float *g0 = F(P->G[0]), *g1 = F(P->G[1]), *g2 = F(P->G[2]);     // g0: gradient w.r.t. the current block output
    RUN(dsspk_gap_bwd(s, F(P->dpooled), g0, m, 64, 64));
    // Per convolution layer the backward pass is  BN backward -> d-input convolution -> d-filter convolution.
    // Where the specialised 3x3 kernels apply, and the gradient arrives already masked with sum records (written by the
    // epilogue of the d-input convolution before it), these collapse (regular_layer below):
    //   stages 1-2: ONE kernel - BN backward in its loader, d-input convolution, ReLU mask + sum records of the
    //               next batch norm in its epilogue, and the d-filter partial sums from the same LDS tiles (dx is
    //               never stored) - followed by the small kernel that sums those records
    //   stage 3   : the d-input kernel (stores dx), then the d-filter kernel, which carries the sums job
    // In both forms the d-input kernel carries the reduction of the PREVIOUS layer's d-filter partial sums, which
    // therefore alternate between two scratch buffers.
    // Everything else (first and last layers, the stride-2 blocks) takes the stand-alone kernels.
    //   parts0 > 0 : g0 holds the masked dz of this block's BN2 and recB0 its records
    //   tot0       : their sums are in totB already (and dgamma / dbeta of BN2 stored)
    //   pend       : d-filter partial sums whose reduction has not been launched yet
    float *recB0 = F(P->bn_scratch2), *totA = F(P->tot_a), *totB = F(P->tot_b);
    float* scrs[2] = {scr, F(P->wg_scratch2)};
    int parts0 = 0;
    bool tot0 = false;
    struct { float* partial; float* dw; int E, chunks; bool on; } pend = {nullptr, nullptr, 0, 0, false};
    auto flush = [&]() -> int {
        if (!pend.on) return 0;
        pend.on = false;
        return dsspk_wgrad_reduce(s, pend.partial, pend.dw, pend.E, pend.chunks);
    };
    // dz (masked, records summed into tot) -> through BN (xc, st, gamma) -> dx -> d-input (+ add) with the mask / records
    // epilogue (mask_src = x_in, xc_post, st_post -> records) into out, and d-filter (x_in, dx) into dw (pending).
    // nrec != NULL: the records just written are summed into ntot / ndgamma / ndbeta for the next layer.
    auto regular_layer = [&](const float* dz, const float* xc, const float* st, const float* gamma, const float* tot,
                             const float* wt, const float* add, float* out, const float* x_in, const float* xc_post,
                             const float* st_post, float* records, float* dw, int H, int Cc, bool sum_next, int nparts,
                             float* ntot, float* ndgamma, float* ndbeta) -> int {
        float* out_scr = (pend.on && pend.partial == scrs[0]) ? scrs[1] : scrs[0];
        const float* rp = pend.on ? pend.partial : nullptr;
        int chunks = dsspk_conv_bwd_fused_chunks(m, H, Cc);
        if (chunks > 0) {
            RUN(dsspk_conv_bwd_data_bn_wgrad(s, dz, xc, st, gamma, tot, wt, add, out, xc_post, st_post, records, x_in,
                                             out_scr, rp, pend.dw, pend.E, pend.chunks, m, H, Cc));
            if (sum_next) RUN(dsspk_bn_bwd_totals(s, records, nparts, Cc, ntot, ndgamma, ndbeta));
        } else {
            RUN(dsspk_conv_bwd_data_bn(s, dz, xc, st, gamma, tot, g1, wt, add, out, x_in, xc_post, st_post, records,
                                       rp, pend.dw, pend.E, pend.chunks, m, H, Cc));
            RUN(dsspk_conv_bwd_weight_parts(s, x_in, g1, out_scr, m, H, H, Cc, Cc, 3, 3, 1, 1, sum_next ? records : nullptr,
                                            nparts, Cc, ntot, ndgamma, ndbeta, &chunks));
        }
        pend.partial = out_scr; pend.dw = dw; pend.E = 9 * Cc * Cc; pend.chunks = chunks; pend.on = true;
        return 0;
    };
    for (int bi = (int)P->blocks.size() - 1; bi >= 0; --bi) {
        const ResBlock& B = P->blocks[bi];
        const float* xin = bi ? F(P->blocks[bi - 1].out) : F(P->stem_a);
        const int Ho = B.H / B.stride;
        const long M = (long)m * Ho * Ho;
        const int parts1 = dsspk_conv_fwd_stat_parts(m, Ho, Ho, B.cout, B.cout, 3, 3, 1, 1);
        const bool identity = B.stride == 1 && B.cin == B.cout;
        const int partsp = identity ? dsspk_conv_fwd_stat_parts(m, B.H, B.H, B.cin, B.cout, 3, 3, 1, 1) : 0;
        const bool fused1 = parts1 > 0 && partsp > 0;        // conv1's layer takes the two-launch form
        bool tot1 = false;                                   // sums of BN1's records are in totA
        // ---- BN2 + conv2: g0 = dz2 -> g1 = d conv2 output, g2 = dz1 = d a1 * [a1 > 0] (+ BN1's records in bscr)
        if (parts0 > 0 && parts1 > 0) {
            if (!tot0) RUN(dsspk_bn_bwd_totals(s, recB0, parts0, B.cout, totB, g + B.g2, g + B.b2));
            RUN(regular_layer(g0, F(B.c2), F(B.st2), w + B.g2, totB, w + B.w2, nullptr, g2, F(B.a1), F(B.c1), F(B.st1), bscr,
                              g + B.w2, Ho, B.cout, fused1, parts1, totA, g + B.g1, g + B.b1));
            tot1 = fused1;
        } else {
            RUN(flush());
            if (!parts0) RUN(dsspk_bn_bwd_reduce(s, F(B.c2), F(B.st2), g0, F(B.out), recB0, M, B.cout));
            RUN(dsspk_bn_bwd_dx(s, F(B.c2), w + B.g2, F(B.st2), g0, g1, g + B.g2, g + B.b2, recB0, M, B.cout, parts0));
            RUN(dsspk_conv_bwd_weight(s, F(B.a1), g1, g + B.w2, scr, m, Ho, Ho, B.cout, B.cout, 3, 3, 1, 1));
            if (parts1) {
                RUN(dsspk_conv_bwd_data_post(s, g1, w + B.w2, nullptr, g2, F(B.a1), F(B.c1), F(B.st1), bscr, m, Ho, B.cout));
            } else {
                RUN(dsspk_conv_bwd_data(s, g1, w + B.w2, nullptr, g2, m, Ho, Ho, B.cout, B.cout, 3, 3, 1, 1));
                RUN(dsspk_bn_bwd_reduce(s, F(B.c1), F(B.st1), g2, F(B.a1), bscr, M, B.cout));
            }
        }
        // ---- BN1 + conv1: g2 = dz1 -> g1 = d conv1 output; d-input (+ dz2 through an identity shortcut) = gradient
        //      w.r.t. the block's input, which is the previous block's (or the stem's) post-ReLU output: mask +
        //      records of ITS batch norm in the same kernel where the specialised kernel applies
        if (fused1) {
            const float* pc = bi ? F(P->blocks[bi - 1].c2) : F(P->stem_c);
            const float* pst = bi ? F(P->blocks[bi - 1].st2) : F(P->stem_st);
            if (!tot1) RUN(dsspk_bn_bwd_totals(s, bscr, parts1, B.cout, totA, g + B.g1, g + B.b1));
            // output in place over the shortcut's gradient g0; g0 stays the gradient w.r.t. the previous block's output
            const bool next_fused = bi > 0;                  // the previous block's conv2 has this convolution's shape
            RUN(regular_layer(g2, F(B.c1), F(B.st1), w + B.g1, totA, w + B.w1, g0, g0, xin, pc, pst, recB0, g + B.w1, B.H, B.cin,
                              next_fused, partsp, totB, next_fused ? g + P->blocks[bi - 1].g2 : nullptr,
                              next_fused ? g + P->blocks[bi - 1].b2 : nullptr));
            parts0 = partsp;
            tot0 = next_fused;
        } else {
            RUN(flush());
            RUN(dsspk_bn_bwd_dx(s, F(B.c1), w + B.g1, F(B.st1), g2, g1, g + B.g1, g + B.b1, bscr, M, B.cout, parts1));
            RUN(dsspk_conv_bwd_weight(s, xin, g1, g + B.w1, scr, m, B.H, B.H, B.cin, B.cout, 3, 3, B.stride, 1));
            if (partsp) {
                const float* pc = bi ? F(P->blocks[bi - 1].c2) : F(P->stem_c);
                const float* pst = bi ? F(P->blocks[bi - 1].st2) : F(P->stem_st);
                RUN(dsspk_conv_bwd_data_post(s, g1, w + B.w1, g0, g2, xin, pc, pst, recB0, m, B.H, B.cin));
            } else {
                RUN(dsspk_conv_bwd_data(s, g1, w + B.w1, identity ? g0 : nullptr, g2, m, B.H, B.H, B.cin, B.cout, 3, 3, B.stride, 1));
                if (!identity) RUN(dsspk_shortcut_bwd_acc(s, g0, g2, m, Ho, Ho, B.cout));
            }
            parts0 = partsp;
            tot0 = false;
            float* t = g0; g0 = g2; g2 = t;
        }
    }
    RUN(flush());
    if (!parts0) RUN(dsspk_bn_bwd_reduce(s, F(P->stem_c), F(P->stem_st), g0, F(P->stem_a), recB0, (long)m * 1024, 16));
    RUN(dsspk_bn_bwd_dx(s, F(P->stem_c), w + P->stem_g, F(P->stem_st), g0, g1, g + P->stem_g, g + P->stem_b, recB0,
                        (long)m * 1024, 16, parts0));
    RUN(dsspk_conv_bwd_weight(s, x, g1, g + P->stem_w, scr, m, 32, 32, 3, 16, 3, 3, 1, 1));
    return 0;
}

}  // namespace

Plan* create(int model_id, int batch, int n_classes, int K, void* workspace_dev, std::string& err) {
    Plan* P = new Plan();
    if (!P->build(model_id, batch, n_classes)) { err = "unknown model"; delete P; return nullptr; }
    if (batch > 1024 || n_classes > 1024) { err = "batch and n_classes must be <= 1024"; delete P; return nullptr; }
    P->K = K;
    P->ws = (char*)workspace_dev;
    return P;
}

void destroy(Plan* p) { delete p; }

int step(Plan* P, int worker, hipStream_t stream, const float* x, const int32_t* y, const float* w, float* g, float* loss,
         std::string& err) {
    char* ws = P->ws + (size_t)worker * P->per_worker;
    if (P->model_id == DSSP_MODEL_MLP) return step_mlp(P, ws, stream, x, y, w, g, loss, err);
    if (P->model_id == DSSP_MODEL_ALEXNET_DS) return step_alexnet(P, ws, stream, x, y, w, g, loss, err);
    if (P->model_id == DSSP_MODEL_ALEXNET_3C) return step_alexnet3(P, ws, stream, x, y, w, g, loss, err);
    return step_resnet(P, ws, stream, x, y, w, g, loss, err);
}

}  // namespace dssp_model

extern "C" int64_t dssp_model_param_count(int model_id, int n_classes) {
    dssp_model::Plan P;
    if (n_classes < 2 || !P.build(model_id, 1, n_classes)) return -1;
    return P.n_params;
}

extern "C" int dssp_model_segments(int model_id, int n_classes, int32_t* kind, int64_t* size, int64_t* fan_in, int max_segments) {
    dssp_model::Plan P;
    if (n_classes < 2 || !P.build(model_id, 1, n_classes)) return DSSP_EINVAL;
    const int n = (int)P.segs.size();
    for (int i = 0; i < n && i < max_segments; ++i) {
        if (kind) kind[i] = P.segs[i].kind;
        if (size) size[i] = P.segs[i].size;
        if (fan_in) fan_in[i] = P.segs[i].fan_in;
    }
    return n;
}

extern "C" size_t dssp_workspace_bytes(int model_id, int batch, int n_classes, int K) {
    dssp_model::Plan P;
    if (model_id == DSSP_MODEL_NONE) return 0;
    if (n_classes < 2 || batch < 1 || K < 1 || !P.build(model_id, batch, n_classes)) return 0;
    return P.per_worker * (size_t)K;
}

extern "C" int dssp_workspace_tensor(int model_id, int batch, int n_classes, int K, int worker, int what, int index,
                                     size_t* byte_offset, int64_t* count) {
    dssp_model::Plan P;
    if (n_classes < 2 || batch < 1 || worker < 0 || worker >= K || !P.build(model_id, batch, n_classes)) return DSSP_EINVAL;
    int seen = 0;
    for (const auto& t : P.tens)
        if (t.what == what) {
            if (seen == index) {
                if (byte_offset) *byte_offset = (size_t)worker * P.per_worker + t.off;
                if (count) *count = t.count;
                return DSSP_OK;
            }
            ++seen;
        }
    return DSSP_EINVAL;
}
