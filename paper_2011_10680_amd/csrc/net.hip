// Whole-network plan for the integer-only ResNet18 / ResNet50 forward (Figure 2, Section 3.3):
// topology, storage rule for mixed precision, workspace slot assignment, parameter arena (weights also in the
// implicit-GEMM kernel's blocked order) and the launch sequence (a large batch as two parts on two streams).
// Host code only; the kernels live in the other translation units.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

// Workspace of hawq_forward_resnet_noalloc: a fixed array in device memory that belongs to the library's code object (one
// copy per GPU the library is loaded on, held until the process ends).  In host code this name is only a handle for
// hipGetSymbolAddress -- never an address a kernel could use; the per-device address is resolved once (scratch_base below)
// and that pointer is what reaches the kernels, exactly as a caller's workspace pointer does.
#define HAWQ_NOALLOC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[HAWQ_NOALLOC_SCRATCH_BYTES];

namespace hawq {
hawq_status make_conv_args(const hawq_conv_desc *d, const void *x, const void *w, const int32_t *bias, const int32_t *b,
                           const uint8_t *c, const void *residual, const int32_t *res_b, const uint8_t *res_c, void *y,
                           bool check_pointers, ConvArgs &a, int &x_hi_out);
hawq_status dispatch_conv(const ConvArgs &a, int x_hi, hipStream_t s);
hawq_status make_dual_args(const hawq_conv_desc *d, const void *x, const void *w, const int32_t *bias, const int32_t *b,
                           const uint8_t *c, const hawq_conv_desc *ds, const void *xs, const void *ws, const int32_t *bias_s,
                           const int32_t *b_s, const uint8_t *c_s, void *y, bool check_pointers, ConvArgs &a, int &x_hi, int &xs_hi);
hawq_status dispatch_conv_dual(const ConvArgs &a, int x_hi, int xs_hi, hipStream_t s);
void stem_pack_weights(const int8_t *w, int8_t *out);
bool conv_stem_eligible(const ConvArgs &a);
}  // namespace hawq

using namespace hawq;

namespace {

struct LayerShape {
    std::string name;
    int C, K, R, S, stride, pad, H, W, P, Q;
    bool has_residual, is_ds, is_c1, is_fc, is_stem;
    int block;  // running block index, -1 for stem / fc
};

int conv_out(int h, int r, int s, int p) { return (h + 2 * p - r) / s + 1; }

// Canonical layer list: conv1; per block c1, c2, [c3], [ds]; fc.
bool build_topology(int arch, int hw, int classes, std::vector<LayerShape> &out) {
    static const int widths[4] = {64, 128, 256, 512};
    int depth18[4] = {2, 2, 2, 2}, depth50[4] = {3, 4, 6, 3};
    const int *depth = arch == 18 ? depth18 : (arch == 50 ? depth50 : nullptr);
    if (!depth || hw < 32 || classes <= 0) return false;
    out.clear();
    int p1 = conv_out(hw, 7, 2, 3);
    out.push_back({"conv1", 3, 64, 7, 7, 2, 3, hw, hw, p1, p1, false, false, false, false, true, -1});
    int h = conv_out(p1, 3, 2, 1);
    int cin = 64, blk = 0;
    for (int si = 0; si < 4; ++si)
        for (int bi = 0; bi < depth[si]; ++bi, ++blk) {
            const int wd = widths[si], s = (si > 0 && bi == 0) ? 2 : 1;
            const int cout = wd * (arch == 50 ? 4 : 1);
            const int ho = conv_out(h, 1, s, 0);
            char pre[32];
            snprintf(pre, sizeof pre, "layer%d.%d", si + 1, bi);
            const std::string n(pre);
            if (arch == 50) {
                out.push_back({n + ".c1", cin, wd, 1, 1, s, 0, h, h, ho, ho, false, false, true, false, false, blk});
                out.push_back({n + ".c2", wd, wd, 3, 3, 1, 1, ho, ho, ho, ho, false, false, false, false, false, blk});
                out.push_back({n + ".c3", wd, cout, 1, 1, 1, 0, ho, ho, ho, ho, true, false, false, false, false, blk});
            } else {
                out.push_back({n + ".c1", cin, wd, 3, 3, s, 1, h, h, ho, ho, false, false, true, false, false, blk});
                out.push_back({n + ".c2", wd, cout, 3, 3, 1, 1, ho, ho, ho, ho, true, false, false, false, false, blk});
            }
            if (s != 1 || cin != cout)
                out.push_back({n + ".ds", cin, cout, 1, 1, s, 0, h, h, ho, ho, false, true, false, false, false, blk});
            cin = cout;
            h = ho;
        }
    out.push_back({"fc", cin, classes, 1, 1, 1, 0, 1, 1, 1, 1, false, false, false, true, false, -1});
    return true;
}

// STEP_CONV_DUAL: a block's last convolution and its transition convolution in one launch (both INT32 accumulators
// rescaled and added); STEP_RESADD: the same sum formed from two raw INT32 tensors in the workspace.
enum StepKind { STEP_STEM, STEP_MAXPOOL, STEP_CONV, STEP_AVGPOOL, STEP_FC, STEP_CONV_DUAL, STEP_RESADD };

struct Tensor {           // a stored activation
    int64_t elems_per_image;
    int dt;
    int dims[3];          // P, Q, K
    int slot = -1;
    int last_use = -1;    // last step that reads it
};

struct Step {
    StepKind kind;
    std::string name;
    int layer = -1;               // index into the canonical layer list
    int in = -1, res = -1, out = -1;  // tensor ids (-1: external image / logits)
    hawq_conv_desc desc{};        // N filled per call
    hawq_conv_desc desc_s{};      // STEP_CONV_DUAL: the transition convolution (reads tensor `res`)
    const uint8_t *w_s = nullptr;             // ... its parameters
    const uint8_t *w_t = nullptr, *w_s_t = nullptr;   // the weights (and the shortcut's) in the implicit-GEMM kernel's blocked order
    const uint8_t *w_s_f = nullptr;                   // the shortcut's in fragment order
    bool dual16 = false;   // two-convolution launches (STEP_CONV_DUAL, fused pairs): the main branch's rescaled term provably fits 16 bits
    const int32_t *bias_s = nullptr, *b_s = nullptr;
    const uint8_t *c_s = nullptr;
    bool raw = false;             // STEP_CONV: store the INT32 accumulator + bias, no requantisation
    // A transition convolution and the block's last convolution that adds its output (stored-shortcut form): where the
    // two-convolution kernels apply, the pair runs as one launch at the last convolution's step, with the
    // transition tensor's rounding done in registers -- same bits, no round trip, and the transition step launches nothing.
    int pair_last = -1;           // on the transition step: index of the last convolution's step
    int pair_ds = -1;             // on the last convolution's step: index of the transition step
    const uint8_t *w = nullptr;   // device parameter pointers
    const uint8_t *w_stem = nullptr;      // conv1 only: weights re-tiled for the stem kernel
    const int32_t *bias_stem = nullptr;   //             bias + 128 * sum(w) (input offset correction)
    const int32_t *bias = nullptr, *b = nullptr, *res_b = nullptr;
    const uint8_t *c = nullptr, *res_c = nullptr;
    double macs_per_image = 0, bytes_per_image = 0, bytes_fixed = 0;
    const uint8_t *w_f = nullptr; // the weights in MFMA fragment order (resident-pixel 3x3 kernel and its fused 1x1), or null
    // A bottleneck's 3x3 convolution and the 1x1 convolution + shortcut that follows it as one launch (the tensor between
    // them is never stored): the 3x3 step launches nothing (tail_next = index of the 1x1 step), the 1x1 step launches both
    // (tail_prev = index of the 3x3 step).
    int tail_next = -1, tail_prev = -1;
    bool fused_pool = false;      // conv1 step: the max pool is computed in the same kernel (writes the pool's tensor)
    bool skip = false;            // max-pool step when conv1 has absorbed it: nothing to launch
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Device address of `scratch` on the current device, resolved on first use per device (hawq_net_create does it for the
// device the network is created on, so the forward itself normally finds it cached).  nullptr if a HIP call fails.
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;
void *scratch_base() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

struct hawq_net {
    int arch, hw, classes, keep;
    std::vector<LayerShape> layers;
    std::vector<Tensor> tensors;
    std::vector<Step> steps;
    std::vector<int64_t> slot_bytes_per_image;
    void *arena = nullptr;
    // a large batch runs as two parts on two streams (see hawq_forward_resnet): the second stream and the fork / join events
    hipStream_t aux_stream = nullptr;
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
};

namespace {

int act_hi(int bits) { return bits == 8 ? 127 : 15; }

// Assign workspace slots: a tensor's slot is free again after its last reader has run.
void assign_slots(hawq_net *net) {
    auto &T = net->tensors;
    for (size_t s = 0; s < net->steps.size(); ++s) {
        const Step &st = net->steps[s];
        if (st.in >= 0) T[st.in].last_use = (int)s;
        if (st.res >= 0) T[st.res].last_use = (int)s;
        // a transition step that is carried out at its block's last convolution reads its input there
        if (st.pair_ds >= 0 && net->steps[st.pair_ds].in >= 0) T[net->steps[st.pair_ds].in].last_use = (int)s;
        // likewise the input of a 3x3 convolution that runs inside its successor's launch
        if (st.tail_prev >= 0 && net->steps[st.tail_prev].in >= 0) T[net->steps[st.tail_prev].in].last_use = (int)s;
    }
    std::vector<int> owner;  // slot -> tensor currently in it (-1 free)
    auto &sb = net->slot_bytes_per_image;
    sb.clear();
    for (size_t s = 0; s < net->steps.size(); ++s) {
        const Step &st = net->steps[s];
        if (st.out < 0) continue;
        Tensor &t = T[st.out];
        const int64_t need = tensor_bytes(t.elems_per_image, t.dt);
        int pick = -1;
        if (!net->keep) {
            for (size_t i = 0; i < owner.size(); ++i) {
                if (owner[i] >= 0 && T[owner[i]].last_use < (int)s) owner[i] = -1;  // dead before this step
            }
            // best fit among free slots, else the largest free one (it grows), else a new slot
            int64_t best = -1;
            for (size_t i = 0; i < owner.size(); ++i)
                if (owner[i] < 0 && sb[i] >= need && (best < 0 || sb[i] < best)) { best = sb[i]; pick = (int)i; }
            if (pick < 0)
                for (size_t i = 0; i < owner.size(); ++i)
                    if (owner[i] < 0 && (pick < 0 || sb[i] > sb[pick])) pick = (int)i;
        }
        if (pick < 0) { owner.push_back(-1); sb.push_back(0); pick = (int)owner.size() - 1; }
        owner[pick] = st.out;
        if (sb[pick] < need) sb[pick] = need;
        t.slot = pick;
    }
}

// Does the (transition, last convolution) pair whose transition step is `ds_step` run as one launch at batch N?
bool pair_runs_fused(const hawq_net *net, int N, int ds_step) {
    const Step &d = net->steps[ds_step];
    if (d.pair_last < 0 || net->keep) return false;
    (void)N;
    // A 3x3 main convolution (ResNet18) in the four-wave two-accumulator kernel runs slower than as two launches: that
    // kernel is a third slower per multiply-accumulate than the plain one, and a 3x3 convolution is all
    // multiply-accumulates (7x7, 512 -> 512 at batch 64: 37 us as one launch, 8 + 18 us as two).  One launch only where
    // the eight-wave 16-bit form applies (ResNet18 batch 64, stored form: 189 k four-wave, 202 k two launches, 210 k).
    if (net->steps[d.pair_last].desc.R == 3 && !net->steps[d.pair_last].dual16) return false;
    return true;   // 8-bit operands on both branches (checked when the plan was made): one of the two-convolution kernels applies
}

size_t slot_offset(const hawq_net *net, int slot, int N) {
    size_t off = 0;
    for (int i = 0; i < slot; ++i) off += align_up((size_t)net->slot_bytes_per_image[i] * N, 256);
    return off;
}

size_t workspace_one_part(const hawq_net *net, int N) { return slot_offset(net, (int)net->slot_bytes_per_image.size(), N); }

// Batch split.  Every kernel of a forward pays a ramp-up and a tail in which part of the chip idles (tiles do not divide
// evenly over 256 CUs, pipelines fill and drain), about a fifth of a ResNet50 forward at batch 128.  Images are
// independent, so a large batch is run as two parts on two streams: the second part's kernels fill the first part's
// gaps (measured 5 % on ResNet50 at batch 128 with equal parts; nothing at batch 64, a loss with three or four parts).
// Returns the size of the first part, 0 for no split.
int g_split_override = 0;   // 0: rule below; -1: never split; n > 0: first part of n images (measurement hook)
int g_fuse_tails = 0;       // networks created from now on: 0 = the plan's rule for fused bottleneck tails, 1 = wherever the kernel applies, -1 = nowhere
int split_first_part(const hawq_net *net, int N) {
    if (net->keep || !net->aux_stream) return 0;
    if (g_split_override < 0) return 0;
    int n1 = ((N / 2) + 7) & ~7;
    if (g_split_override > 0) n1 = g_split_override;
    else if (N < 96) return 0;
    if (n1 >= N) return 0;
    // the second part's images start n1 images into the batch: conv1's kernel wants that address 16-byte aligned
    if (((size_t)n1 * net->hw * net->hw * 3) % 16 != 0) return 0;
    return n1;
}

}  // namespace

extern "C" {

int32_t hawq_net_num_layers(int32_t arch) {
    std::vector<LayerShape> L;
    return build_topology(arch, 224, 1000, L) ? (int32_t)L.size() : 0;
}

hawq_status hawq_net_layer_info(int32_t arch, int32_t image_hw, int32_t num_classes, int32_t index, hawq_layer_info *out) {
    if (!out) return HAWQ_ERR_NULL;
    std::vector<LayerShape> L;
    if (!build_topology(arch, image_hw, num_classes, L)) return HAWQ_ERR_SHAPE;
    if (index < 0 || index >= (int)L.size()) return HAWQ_ERR_RANGE;
    const LayerShape &l = L[index];
    memset(out, 0, sizeof *out);
    snprintf(out->name, sizeof out->name, "%s", l.name.c_str());
    out->C = l.C; out->K = l.K; out->R = l.R; out->S = l.S; out->stride = l.stride; out->pad = l.pad;
    out->H = l.H; out->W = l.W; out->P = l.P; out->Q = l.Q;
    out->has_residual = l.has_residual; out->is_ds = l.is_ds;
    return HAWQ_OK;
}

hawq_status hawq_net_create(int32_t arch, int32_t image_hw, int32_t num_classes, const hawq_layer_params *lp, int32_t n_layers,
                            const int32_t *pool_b, const uint8_t *pool_c, int32_t keep_activations, hawq_net **out) {
    if (!lp || !pool_b || !pool_c || !out) return HAWQ_ERR_NULL;
    *out = nullptr;
    hawq_net *net = new hawq_net();
    net->arch = arch; net->hw = image_hw; net->classes = num_classes; net->keep = keep_activations != 0;
    if (!build_topology(arch, image_hw, num_classes, net->layers)) { delete net; return HAWQ_ERR_SHAPE; }
    auto &L = net->layers;
    const int nl = (int)L.size();
    if (n_layers != nl) { delete net; return HAWQ_ERR_SHAPE; }
    auto fail = [&](hawq_status st) { hawq_net_destroy(net); return st; };   // (frees whatever has been created so far)

    // ---- validate parameters (host data: ranges can be checked here) ----
    for (int i = 0; i < nl; ++i) {
        const hawq_layer_params &p = lp[i];
        if (!p.w || !p.bias) return fail(HAWQ_ERR_NULL);
        if (!L[i].is_fc && (!p.b || !p.c)) return fail(HAWQ_ERR_NULL);
        if (p.flags & ~HAWQ_LAYER_INT32_SHORTCUT) return fail(HAWQ_ERR_UNSUPPORTED);
        if ((p.flags & HAWQ_LAYER_INT32_SHORTCUT) && !L[i].is_ds) return fail(HAWQ_ERR_UNSUPPORTED);
        // the shortcut multiplier of a block's last convolution is unused when its transition layer keeps INT32
        const bool i32sc = L[i].has_residual && i + 1 < nl && L[i + 1].is_ds && (lp[i + 1].flags & HAWQ_LAYER_INT32_SHORTCUT);
        if (L[i].has_residual && !i32sc && (!p.res_b || !p.res_c)) return fail(HAWQ_ERR_NULL);
        if (p.bits != 4 && p.bits != 8) return fail(HAWQ_ERR_DTYPE);
        if ((L[i].is_stem || L[i].is_fc) && p.bits != 8) return fail(HAWQ_ERR_DTYPE);
        if (L[i].is_ds) {
            int j = i;
            while (j >= 0 && !(L[j].is_c1 && L[j].block == L[i].block)) --j;
            if (j < 0 || lp[j].bits != p.bits) return fail(HAWQ_ERR_DTYPE);
        }
        if (!L[i].is_fc)
            for (int k = 0; k < L[i].K; ++k) {
                if (p.b[k] < 0 || p.c[k] < 1 || p.c[k] > 62) return fail(HAWQ_ERR_RANGE);
                if (L[i].has_residual && !i32sc && (p.res_b[k] < 0 || p.res_c[k] < 1 || p.res_c[k] > 62)) return fail(HAWQ_ERR_RANGE);
            }
    }
    const int c_last = L[nl - 1].C;
    for (int k = 0; k < c_last; ++k)
        if (pool_b[k] < 0 || pool_c[k] < 1 || pool_c[k] > 62) return fail(HAWQ_ERR_RANGE);

    // ---- 4-bit layers that run in expanded form ----
    // There is no 4-bit matrix instruction: a 4-bit layer saves bytes, not multiply-accumulates, and the streaming kernels
    // (1x1 with few input channels, the 64-channel 3x3) are the ones that profit.  Everywhere else the network keeps a
    // 4-bit layer's input in an 8-bit container (values 0..15, written so by the producer's epilogue) and its weights expanded
    // to INT8 in the arena, and the layer runs on the INT8 kernels at INT8 speed -- same integers, other storage.  A block's
    // transition layer and first convolution read the same tensor and go together; in a block with a transition layer
    // the last convolution and the transition layer are expanded so that they can run as one launch.  With kept
    // activations every tensor stays in the documented packed form.
    std::vector<char> expand(nl, 0);
    if (!net->keep) {
        auto packed_pays = [&](const LayerShape &l) {
            const bool pw = l.R == 1 && l.S == 1 && (l.C == 64 || l.C == 128 || (l.C == 256 && l.K <= 128));
            const bool c64 = l.R == 3 && l.S == 3 && l.C == 64 && l.K == 64 && l.stride == 1 && l.pad == 1;
            // packed LDS-DMA form of the implicit-GEMM kernel.  (Running these layers in 8-bit form on the resident-pixel
            // kernel instead was measured on the mixed network at batch 256: the 3x3 layer gains nothing there -- 45.7 against
            // 46.2 us at 28x28 -- and its producer writes twice the bytes, 36 against 30 us.)
            const bool c128 = l.R == 3 && l.S == 3 && l.C % 128 == 0;
            return pw || c64 || c128;
        };
        for (int i = 0; i < nl; ++i)
            if (lp[i].bits == 4 && !L[i].is_stem && !L[i].is_fc) expand[i] = !packed_pays(L[i]);
        for (int i = 0; i < nl; ++i) {
            if (!L[i].is_ds || lp[i].bits != 4) continue;
            int c1 = i, last = i;
            while (c1 >= 0 && !(L[c1].is_c1 && L[c1].block == L[i].block)) --c1;
            while (last >= 0 && !(L[last].has_residual && L[last].block == L[i].block)) --last;
            expand[i] = 1;
            if (c1 >= 0) expand[c1] = 1;                              // (same width as the transition layer: validated above)
            if (last >= 0 && lp[last].bits == 4) expand[last] = 1;
        }
    }
    auto is8 = [&](int i) { return lp[i].bits == 8 || expand[i]; };      // operands in 8-bit form
    auto cont_dt = [&](int i) { return is8(i) ? HAWQ_U8 : HAWQ_U4; };     // container of the tensor layer i reads

    // ---- parameter arena layout ----
    struct Off { size_t w, wt, wf, bias, b, c, rb, rc; };
    // row of the [K][R*S*C] weight matrix in bytes as stored, and whether a blocked copy is made for the implicit-GEMM
    // kernel (64-byte K-steps: 8-bit form with C % 64 == 0, packed 4-bit form with C % 128 == 0)
    auto wrow = [&](int i) { return (int64_t)tensor_bytes((int64_t)L[i].R * L[i].S * L[i].C, is8(i) ? HAWQ_S8 : HAWQ_S4); };
    auto blocked = [&](int i) { return !L[i].is_stem && L[i].C % (is8(i) ? 64 : 128) == 0; };
    // fragment-ordered copy: the 3x3 / 1 / 1 layers the resident-pixel kernel takes (128 or 256 input channels, 8-bit form)
    // and the 1x1 layer that follows such a layer in a bottleneck (it may run fused behind it)
    auto rp3x3 = [&](int i) { return L[i].R == 3 && L[i].S == 3 && L[i].stride == 1 && L[i].pad == 1 && is8(i) && (L[i].C == 128 || L[i].C == 256 || (L[i].C == 512 && L[i].W <= 14)) && L[i].K % L[i].C == 0; };
    // ... and the same layers with packed 4-bit operands (the kernel's packed form)
    auto rp3x3pk = [&](int i) { return L[i].R == 3 && L[i].S == 3 && L[i].stride == 1 && L[i].pad == 1 && !is8(i) && L[i].W <= 28 && (L[i].C == 128 || L[i].C == 256 || (L[i].C == 512 && L[i].W <= 14)) && L[i].K % L[i].C == 0; };
    // ... and the 1x1 layers of the resident-pixel 1x1 kernel (main branches and transition convolutions alike)
    auto rp1x1 = [&](int i) { return L[i].R == 1 && L[i].S == 1 && L[i].pad == 0 && is8(i) && L[i].K % 256 == 0 && (L[i].C == 256 || L[i].C == 512 || L[i].C == 1024 || L[i].C == 2048); };
    auto fragmented = [&](int i) {
        if (L[i].is_stem || L[i].is_fc) return false;
        if (rp3x3(i) || rp3x3pk(i) || rp1x1(i)) return true;
        return i > 0 && L[i].R == 1 && L[i].has_residual && is8(i) && rp3x3(i - 1) && L[i - 1].block == L[i].block && L[i].C == L[i - 1].K;
    };
    std::vector<Off> off(nl);
    size_t total = 0;
    auto take = [&](size_t bytes) { size_t o = total; total = align_up(total + bytes, 256); return o; };
    for (int i = 0; i < nl; ++i) {
        const int64_t nw = (int64_t)L[i].K * L[i].R * L[i].S * L[i].C;
        off[i].w = take((size_t)tensor_bytes(nw, is8(i) ? HAWQ_S8 : HAWQ_S4));
        off[i].wt = blocked(i) ? take((size_t)((L[i].K + 63) / 64) * (size_t)wrow(i) * 64) : 0;
        off[i].wf = fragmented(i) ? take((size_t)((L[i].K + 31) / 32) * 32 * (size_t)L[i].R * L[i].S * L[i].C) : 0;   // (always bytes: 4-bit weights are expanded)
        off[i].bias = take(4 * (size_t)L[i].K);
        off[i].b = take(4 * (size_t)L[i].K);
        off[i].c = take((size_t)L[i].K);
        off[i].rb = take(4 * (size_t)L[i].K);
        off[i].rc = take((size_t)L[i].K);
    }
    const size_t off_pb = take(4 * (size_t)c_last), off_pc = take((size_t)c_last);
    const size_t off_ws = take(64 * 256), off_bs = take(4 * 64);
    std::vector<uint8_t> host(total, 0);
    for (int i = 0; i < nl; ++i) {
        const int64_t nw = (int64_t)L[i].K * L[i].R * L[i].S * L[i].C;
        if (lp[i].bits == 4 && expand[i]) {   // nibbles -> sign-extended bytes (even element in the low nibble)
            const uint8_t *src = (const uint8_t *)lp[i].w;
            int8_t *dst = (int8_t *)&host[off[i].w];
            for (int64_t e = 0; e < nw; ++e) {
                const int v = (src[e >> 1] >> (4 * (e & 1))) & 0xF;
                dst[e] = (int8_t)(v >= 8 ? v - 16 : v);
            }
        } else {
            memcpy(&host[off[i].w], lp[i].w, (size_t)tensor_bytes(nw, lp[i].bits == 4 ? HAWQ_S4 : HAWQ_S8));
        }
        if (blocked(i)) {   // [K][row] -> [K/64][row/64][64][64], rows past K stay zero
            const int64_t row = wrow(i), nsteps = row / 64;
            const uint8_t *src = &host[off[i].w];
            uint8_t *dst = &host[off[i].wt];
            for (int k = 0; k < L[i].K; ++k)
                for (int64_t st = 0; st < nsteps; ++st)
                    memcpy(dst + (((int64_t)(k >> 6) * nsteps + st) * 64 + (k & 63)) * 64, src + k * row + st * 64, 64);
        }
        if (fragmented(i)) {   // [K][row] -> [K/32][row/64][2][64 lanes][16]: see launch_fragment_weights for the order
            const bool four = !is8(i);                 // packed rows: expanded to bytes, even elements of every 32 first
            const int64_t rowp = wrow(i), nsteps = (four ? 2 * rowp : rowp) / 64;
            const uint8_t *src = &host[off[i].w];
            uint8_t *dst = &host[off[i].wf];
            for (int g = 0; g < (L[i].K + 31) / 32; ++g)
                for (int64_t st = 0; st < nsteps; ++st)
                    for (int kk = 0; kk < 2; ++kk)
                        for (int lane = 0; lane < 64; ++lane) {
                            const int rho = lane & 31, khalf = lane >> 5;
                            const int k = g * 32 + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3);
                            uint8_t *d = dst + ((((int64_t)g * nsteps + st) * 2 + kk) * 64 + lane) * 16;
                            if (k >= L[i].K) continue;
                            const int64_t ci = st * 4 + kk * 2 + khalf;
                            if (!four) { memcpy(d, src + k * rowp + ci * 16, 16); continue; }
                            const uint8_t *p = src + k * rowp + (ci >> 1) * 16;
                            for (int j = 0; j < 16; ++j) {
                                const int v = (ci & 1) ? (p[j] >> 4) : (p[j] & 0xF);
                                d[j] = (uint8_t)(int8_t)(v >= 8 ? v - 16 : v);
                            }
                        }
        }
        memcpy(&host[off[i].bias], lp[i].bias, 4 * (size_t)L[i].K);
        if (!L[i].is_fc) {
            memcpy(&host[off[i].b], lp[i].b, 4 * (size_t)L[i].K);
            memcpy(&host[off[i].c], lp[i].c, (size_t)L[i].K);
        }
        if (L[i].has_residual && lp[i].res_b && lp[i].res_c) {
            memcpy(&host[off[i].rb], lp[i].res_b, 4 * (size_t)L[i].K);
            memcpy(&host[off[i].rc], lp[i].res_c, (size_t)L[i].K);
        }
    }
    {   // conv1 for the stem kernel: re-tiled weights, bias corrected for the -128 input offset
        const int8_t *w0 = (const int8_t *)lp[0].w;
        stem_pack_weights(w0, (int8_t *)&host[off_ws]);
        int32_t *bs = (int32_t *)&host[off_bs];
        for (int k = 0; k < 64; ++k) {
            int64_t sum = 0;
            for (int i = 0; i < 147; ++i) sum += w0[k * 147 + i];
            bs[k] = (int32_t)(lp[0].bias[k] + 128 * sum);
        }
    }
    memcpy(&host[off_pb], pool_b, 4 * (size_t)c_last);
    memcpy(&host[off_pc], pool_c, (size_t)c_last);
    if (scratch_base() == nullptr) return fail(HAWQ_ERR_DEVICE);   // (address of the fixed workspace on this device, for hawq_forward_resnet_noalloc)
    if (hipMalloc(&net->arena, total) != hipSuccess) return fail(HAWQ_ERR_DEVICE);
    if (hipMemcpy(net->arena, host.data(), total, hipMemcpyHostToDevice) != hipSuccess) return fail(HAWQ_ERR_DEVICE);
    // second stream (default priority) and the events that order it against the caller's stream
    if (hipStreamCreateWithFlags(&net->aux_stream, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&net->fork_ev, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&net->join_ev, hipEventDisableTiming) != hipSuccess)
        return fail(HAWQ_ERR_DEVICE);
    const uint8_t *A = (const uint8_t *)net->arena;

    // ---- steps ----
    auto new_tensor = [&](int P, int Q, int K, int dt) {
        Tensor t;
        t.elems_per_image = (int64_t)P * Q * K; t.dt = dt; t.dims[0] = P; t.dims[1] = Q; t.dims[2] = K;
        net->tensors.push_back(t);
        return (int)net->tensors.size() - 1;
    };
    // bit width of the conv that reads the tensor produced after layer i's block / stem
    auto reader_after = [&](int i) {   // index of that layer, -1 for the pool / fc (8-bit)
        int j = i + 1;
        while (j < nl && L[j].is_ds) ++j;
        return (j >= nl || L[j].is_fc) ? -1 : j;
    };
    auto reader_bits_after = [&](int i) { const int j = reader_after(i); return j < 0 ? 8 : lp[j].bits; };
    auto reader_dt_after = [&](int i) { const int j = reader_after(i); return j < 0 ? (int)HAWQ_U8 : cont_dt(j); };
    // May the eight-wave two-accumulator kernel keep the main branch's rescaled term in 16 bits?  Worst case over all
    // inputs, from the host copies: every multiplier in the narrow evaluation's range and, per output channel,
    // (in_max sum|w| + |bias|) b / 2^c below 32767.  with_res: the stored-shortcut form, whose second rescaling counts too.
    auto fits16 = [&](int last, int ds, int in_bits_main, bool with_res) {
        const int8_t *wm = (const int8_t *)&host[off[last].w];
        const int64_t row = (int64_t)L[last].R * L[last].S * L[last].C;
        auto narrow = [](int32_t b, int c) { return c >= 1 && c <= 32 && ((int64_t)b >> (c - 1)) == 0; };
        for (int k = 0; k < L[last].K; ++k) {
            int64_t sum = 0;
            for (int64_t e = 0; e < row; ++e) sum += wm[k * row + e] < 0 ? -(int64_t)wm[k * row + e] : wm[k * row + e];
            const int64_t bias = lp[last].bias[k];
            const int64_t amax = (int64_t)act_hi(in_bits_main) * sum + (bias < 0 ? -bias : bias);
            const int c = lp[last].c[k];
            if (!narrow(lp[last].b[k], c) || !narrow(lp[ds].b[k], lp[ds].c[k])) return false;
            if (((amax * (int64_t)lp[last].b[k]) >> c) + 2 > 32767) return false;
            if (with_res && (lp[last].res_c[k] > 31 || lp[last].res_b[k] >= (1 << 22))) return false;
        }
        return true;
    };
    auto conv_step = [&](int i, int in_t, int in_dt, int in_hi, int res_t, int res_dt, int out_bits, int out_dt, bool signed_out,
                         bool relu, bool raw = false) {
        Step st;
        st.raw = raw;
        st.kind = L[i].is_stem ? STEP_STEM : STEP_CONV;
        st.name = L[i].name; st.layer = i; st.in = in_t; st.res = res_t;
        hawq_conv_desc &d = st.desc;
        d.N = 1; d.H = L[i].H; d.W = L[i].W; d.C = L[i].C; d.K = L[i].K; d.R = L[i].R; d.S = L[i].S;
        d.stride_h = d.stride_w = L[i].stride; d.pad_h = d.pad_w = L[i].pad;
        d.x_dtype = in_dt; d.w_dtype = is8(i) ? HAWQ_S8 : HAWQ_S4;
        d.y_dtype = signed_out ? HAWQ_S8 : (L[i].is_stem ? (int)HAWQ_U8 : out_dt);
        d.res_dtype = res_dt; d.relu = relu; d.y_lo = signed_out ? -128 : 0; d.y_hi = signed_out ? 127 : act_hi(out_bits);
        if (raw) { d.y_dtype = HAWQ_S32; d.relu = 0; d.y_lo = INT32_MIN; d.y_hi = INT32_MAX; }
        d.x_hi = in_hi;
        st.w = A + off[i].w; st.bias = (const int32_t *)(A + off[i].bias);
        st.w_t = blocked(i) ? A + off[i].wt : nullptr;
        st.w_f = fragmented(i) ? A + off[i].wf : nullptr;
        st.b = (const int32_t *)(A + off[i].b); st.c = A + off[i].c;
        if (res_t >= 0) { st.res_b = (const int32_t *)(A + off[i].rb); st.res_c = A + off[i].rc; }
        st.out = new_tensor(L[i].P, L[i].Q, L[i].K, d.y_dtype);
        const double wbytes = (double)tensor_bytes((int64_t)L[i].K * L[i].R * L[i].S * L[i].C, d.w_dtype);
        st.macs_per_image = (double)L[i].P * L[i].Q * L[i].K * L[i].R * L[i].S * L[i].C;
        // input read once (a strided 1x1 touches only the sampled pixels), output and shortcut once
        const double in_pix = (L[i].R == 1 && L[i].stride > 1) ? (double)L[i].P * L[i].Q : (double)L[i].H * L[i].W;
        st.bytes_per_image = (double)tensor_bytes((int64_t)(in_pix * L[i].C), in_dt) +
                             (double)tensor_bytes((int64_t)L[i].P * L[i].Q * L[i].K, d.y_dtype) +
                             (res_t >= 0 ? (double)tensor_bytes((int64_t)L[i].P * L[i].Q * L[i].K, res_dt) : 0.0);
        st.bytes_fixed = wbytes + 9.0 * L[i].K + (res_t >= 0 ? 5.0 * L[i].K : 0.0);
        net->steps.push_back(st);
        return st.out;
    };

    int li = 0;
    int stage_bits = reader_bits_after(0);
    const int stage_dt = reader_dt_after(0);
    int t = conv_step(0, -1, HAWQ_U8, 255, -1, HAWQ_U8, stage_bits, HAWQ_U8, false, true);
    net->steps[0].w_stem = A + off_ws;
    net->steps[0].bias_stem = (const int32_t *)(A + off_bs);
    {
        Step st;
        st.kind = STEP_MAXPOOL; st.name = "pool"; st.in = t;
        const int P = conv_out(L[0].P, 3, 2, 1);
        st.desc.H = L[0].P; st.desc.W = L[0].Q; st.desc.C = 64; st.desc.x_dtype = HAWQ_U8; st.desc.y_dtype = stage_dt;
        st.desc.y_lo = 0; st.desc.y_hi = act_hi(stage_bits);
        st.out = new_tensor(P, P, 64, stage_dt);
        st.bytes_per_image = (double)L[0].P * L[0].Q * 64 + (double)tensor_bytes((int64_t)P * P * 64, stage_dt);
        // Unless every activation must be kept for inspection, conv1 and the pool run as one kernel and the
        // conv1 tensor is never materialised: it needs no workspace and the pool step launches nothing.
        if (!net->keep && image_hw % 4 == 0) {
            st.skip = true;
            st.bytes_per_image = 0;
            Step &c1 = net->steps[0];
            c1.fused_pool = true;
            net->tensors[c1.out].elems_per_image = 0;
            c1.bytes_per_image = (double)image_hw * image_hw * 3 + (double)tensor_bytes((int64_t)P * P * 64, stage_dt);
        }
        net->steps.push_back(st);
        t = st.out;
    }
    li = 1;
    int in_bits = stage_bits;
    while (li < nl && !L[li].is_fc) {
        // one block: c1, c2, [c3], [ds]
        const int blk = L[li].block;
        std::vector<int> mids;
        int last = -1, ds = -1;
        int j = li;
        for (; j < nl && L[j].block == blk && !L[j].is_fc; ++j) {
            if (L[j].is_ds) ds = j;
            else if (L[j].has_residual) last = j;
            else mids.push_back(j);
        }
        if (lp[mids[0]].bits != in_bits) return fail(HAWQ_ERR_DTYPE);  // cannot happen: in_bits derives from it
        const int out_bits = reader_bits_after(j - 1), out_dt = reader_dt_after(j - 1);
        const int block_in = t, block_in_dt = cont_dt(mids[0]);
        int u = block_in, u_dt = block_in_dt, u_bits = in_bits;
        std::vector<int> chain = mids;
        chain.push_back(last);
        for (size_t q = 0; q < mids.size(); ++q) {
            const int ob = lp[chain[q + 1]].bits;
            u = conv_step(mids[q], u, u_dt, act_hi(u_bits), -1, HAWQ_U8, ob, cont_dt(chain[q + 1]), false, true);
            u_dt = cont_dt(chain[q + 1]); u_bits = ob;
        }
        int sc = block_in, sc_dt = block_in_dt;
        if (ds >= 0 && (lp[ds].flags & HAWQ_LAYER_INT32_SHORTCUT)) {
            // Both branches INT32 (Figure 2).  8-bit operands on both: one launch computes both convolutions and the sum.
            // Otherwise the raw accumulators go through the workspace and a residual-addition launch.
            if (is8(last) && is8(ds)) {
                t = conv_step(last, u, u_dt, act_hi(u_bits), -1, HAWQ_U8, out_bits, out_dt, false, true);
                Step &st = net->steps.back();
                st.kind = STEP_CONV_DUAL;
                st.res = block_in;
                hawq_conv_desc &d = st.desc_s;
                d = st.desc;
                d.H = L[ds].H; d.W = L[ds].W; d.C = L[ds].C; d.R = d.S = 1; d.stride_h = d.stride_w = L[ds].stride; d.pad_h = d.pad_w = 0;
                d.x_dtype = block_in_dt; d.w_dtype = HAWQ_S8; d.x_hi = act_hi(in_bits);   // (8-bit form: block_in_dt is HAWQ_U8)
                st.w_s = A + off[ds].w; st.bias_s = (const int32_t *)(A + off[ds].bias);
                st.w_s_t = blocked(ds) ? A + off[ds].wt : nullptr;
                st.w_s_f = fragmented(ds) ? A + off[ds].wf : nullptr;
                st.dual16 = fits16(last, ds, u_bits, false);
                st.b_s = (const int32_t *)(A + off[ds].b); st.c_s = A + off[ds].c;
                st.macs_per_image += (double)L[ds].P * L[ds].Q * L[ds].K * L[ds].C;
                st.bytes_per_image += (double)L[ds].P * L[ds].Q * L[ds].C;   // a strided 1x1 touches only the sampled pixels
                st.bytes_fixed += (double)L[ds].K * L[ds].C + 9.0 * L[ds].K;
            } else {
                const int r_raw = conv_step(ds, block_in, block_in_dt, act_hi(in_bits), -1, HAWQ_U8, 8, HAWQ_U8, false, false, true);
                const int m_raw = conv_step(last, u, u_dt, act_hi(u_bits), -1, HAWQ_U8, 8, HAWQ_U8, false, false, true);
                net->steps.back().name += ".acc";
                Step st;
                st.kind = STEP_RESADD; st.name = L[last].name; st.layer = last; st.in = m_raw; st.res = r_raw;
                st.desc.H = L[last].P; st.desc.W = L[last].Q; st.desc.K = L[last].K;
                st.desc.y_dtype = out_dt; st.desc.y_lo = 0; st.desc.y_hi = act_hi(out_bits);
                st.b = (const int32_t *)(A + off[last].b); st.c = A + off[last].c;
                st.b_s = (const int32_t *)(A + off[ds].b); st.c_s = A + off[ds].c;
                st.out = new_tensor(L[last].P, L[last].Q, L[last].K, st.desc.y_dtype);
                st.bytes_per_image = 8.0 * L[last].P * L[last].Q * L[last].K +
                                     (double)tensor_bytes((int64_t)L[last].P * L[last].Q * L[last].K, st.desc.y_dtype);
                st.bytes_fixed = 10.0 * L[last].K;
                net->steps.push_back(st);
                t = st.out;
            }
            in_bits = out_bits;
            li = j;
            continue;
        }
        int ds_step = -1;
        if (ds >= 0) {
            sc = conv_step(ds, block_in, block_in_dt, act_hi(in_bits), -1, HAWQ_U8, 8, HAWQ_S8, true, false);
            sc_dt = HAWQ_S8;
            ds_step = (int)net->steps.size() - 1;
        }
        t = conv_step(last, u, u_dt, act_hi(u_bits), sc, sc_dt, out_bits, out_dt, false, true);
        if (ds_step < 0 && !net->keep && mids.size() == 2) {
            // bottleneck with an identity shortcut: 3x3 and the closing 1x1 + shortcut as one launch where the
            // resident-pixel kernel takes the shapes and every tensor involved is in 8-bit form
            const int s3 = (int)net->steps.size() - 1, s2 = s3 - 1;
            Step &c2 = net->steps[s2], &c3 = net->steps[s3];
            RpArgs probe{};
            probe.C = c2.desc.C; probe.K1 = c2.desc.K; probe.K2 = c3.desc.K; probe.H = c2.desc.H; probe.W = c2.desc.W; probe.M = 1;
            const bool types = c2.desc.x_dtype == HAWQ_U8 && c2.desc.y_dtype == HAWQ_U8 && c3.desc.y_dtype == HAWQ_U8 &&
                               c3.desc.res_dtype == HAWQ_U8 && c2.desc.x_hi <= 127;
            // Measured on MI355X at batch 128 (ResNet50 stage 2 / stage 3 shapes): one launch 65 / 39 us, two launches
            // (resident-pixel 3x3, then the streaming 1x1) 55 / 38 us -- the second convolution's integer epilogue binds, and
            // in the fused kernel it runs at two waves per SIMD on the tiles' compute units only.  The plan therefore keeps
            // two launches unless told otherwise (hawq_tune_set_fusion).
            const bool want = g_fuse_tails == 1 || (g_fuse_tails == 2 && c2.desc.C == 256);
            if (want && c2.w_f && c3.w_f && types && c2.desc.R == 3 && c3.desc.R == 1 && conv_rp_shape_ok(probe, true)) {
                c2.tail_next = s3;
                c3.tail_prev = s2;
                net->tensors[c2.out].elems_per_image = 0;   // never stored
            }
        }
        if (ds_step >= 0 && !net->keep && is8(last) && is8(ds)) {
            net->steps[ds_step].pair_last = (int)net->steps.size() - 1;
            net->steps.back().pair_ds = ds_step;
            net->steps.back().dual16 = fits16(last, ds, u_bits, true);
        }
        in_bits = out_bits;
        li = j;
    }
    {
        Step st;
        st.kind = STEP_AVGPOOL; st.name = "avgpool"; st.in = t;
        const LayerShape &pl = L[nl - 2].is_ds ? L[nl - 3] : L[nl - 2];
        st.desc.H = pl.P; st.desc.W = pl.Q; st.desc.C = c_last; st.desc.x_dtype = HAWQ_U8; st.desc.y_dtype = HAWQ_U8;
        st.desc.y_lo = 0; st.desc.y_hi = 127;
        st.b = (const int32_t *)(A + off_pb); st.c = A + off_pc;
        st.out = new_tensor(1, 1, c_last, HAWQ_U8);
        st.bytes_per_image = (double)pl.P * pl.Q * c_last + c_last;
        st.bytes_fixed = 5.0 * c_last;
        net->steps.push_back(st);
        t = st.out;
    }
    {
        const int i = nl - 1;
        Step st;
        st.kind = STEP_FC; st.name = "fc"; st.layer = i; st.in = t;
        hawq_conv_desc &d = st.desc;
        d.N = 1; d.H = 1; d.W = 1; d.C = L[i].C; d.K = L[i].K; d.R = d.S = 1; d.stride_h = d.stride_w = 1;
        d.x_dtype = HAWQ_U8; d.w_dtype = HAWQ_S8; d.y_dtype = HAWQ_S32; d.res_dtype = HAWQ_U8; d.x_hi = 127;
        d.y_lo = INT32_MIN; d.y_hi = INT32_MAX;
        st.w = A + off[i].w; st.bias = (const int32_t *)(A + off[i].bias);
        st.w_t = blocked(i) ? A + off[i].wt : nullptr;
        st.macs_per_image = (double)L[i].C * L[i].K;
        st.bytes_per_image = (double)L[i].C + 4.0 * L[i].K;
        st.bytes_fixed = (double)L[i].C * L[i].K + 4.0 * L[i].K;
        net->steps.push_back(st);
    }
    assign_slots(net);
    *out = net;
    return HAWQ_OK;
}

void hawq_net_destroy(hawq_net *net) {
    if (!net) return;
    if (net->arena) (void)hipFree(net->arena);
    if (net->aux_stream) { (void)hipStreamSynchronize(net->aux_stream); (void)hipStreamDestroy(net->aux_stream); }
    if (net->fork_ev) (void)hipEventDestroy(net->fork_ev);
    if (net->join_ev) (void)hipEventDestroy(net->join_ev);
    delete net;
}

size_t hawq_net_workspace_bytes(const hawq_net *net, int32_t N) {
    if (!net || N <= 0) return 0;
    // room for the batch as one part and as two (256-byte rounding per tensor makes the two layouts differ slightly)
    size_t need = workspace_one_part(net, N);
    const int n1 = split_first_part(net, N);
    if (n1 > 0) {
        const size_t two = workspace_one_part(net, n1) + workspace_one_part(net, N - n1);
        if (two > need) need = two;
    }
    return need;
}

int32_t hawq_net_split_first(const hawq_net *net, int32_t N) { return (net && N > 0) ? split_first_part(net, N) : 0; }

int32_t hawq_net_num_steps(const hawq_net *net) { return net ? (int32_t)net->steps.size() : 0; }

hawq_status hawq_net_step_output(const hawq_net *net, int32_t N, int32_t step, char *name, size_t *offset, size_t *bytes,
                                 int32_t *dtype, int32_t *dims4) {
    if (!net || !name || !offset || !bytes || !dtype || !dims4) return HAWQ_ERR_NULL;
    if (step < 0 || step >= (int)net->steps.size() || N <= 0) return HAWQ_ERR_RANGE;
    const Step &st = net->steps[step];
    snprintf(name, 24, "%s", st.name.c_str());
    if (st.out < 0) {  // fc: the caller's logits
        *offset = 0; *bytes = 0; *dtype = HAWQ_S32;
        dims4[0] = N; dims4[1] = 1; dims4[2] = 1; dims4[3] = net->classes;
        return HAWQ_OK;
    }
    const Tensor &t = net->tensors[st.out];
    *offset = slot_offset(net, t.slot, N);
    *bytes = (size_t)tensor_bytes(t.elems_per_image * N, t.dt);
    *dtype = t.dt;
    dims4[0] = N; dims4[1] = t.dims[0]; dims4[2] = t.dims[1]; dims4[3] = t.dims[2];
    return HAWQ_OK;
}

hawq_status hawq_net_step_cost(const hawq_net *net, int32_t N, int32_t step, double *macs, double *bytes) {
    if (!net || !macs || !bytes) return HAWQ_ERR_NULL;
    if (step < 0 || step >= (int)net->steps.size() || N <= 0) return HAWQ_ERR_RANGE;
    const Step &st = net->steps[step];
    *macs = st.macs_per_image * N;
    *bytes = st.bytes_per_image * N + st.bytes_fixed;
    // a transition / last convolution pair that runs as one launch: all the work and the traffic it still needs (both
    // inputs, both parameter sets, the block output) are reported on the last convolution's step
    if (st.pair_last >= 0 && pair_runs_fused(net, N, step)) { *macs = 0; *bytes = 0; }
    // a 3x3 convolution that runs inside the launch of the 1x1 that follows it: work and traffic (the 3x3's input, the
    // shortcut, the block output, both weight sets) are reported on that step; the tensor in between moves no bytes
    if (st.tail_next >= 0) { *macs = 0; *bytes = 0; }
    if (st.tail_prev >= 0) {
        const Step &p = net->steps[st.tail_prev];
        const double px = (double)st.desc.H * st.desc.W;
        *macs += p.macs_per_image * N;
        *bytes = (px * p.desc.C + 2.0 * px * st.desc.K) * N + st.bytes_fixed + p.bytes_fixed;
    }
    if (st.pair_ds >= 0 && pair_runs_fused(net, N, st.pair_ds)) {
        const Step &d = net->steps[st.pair_ds];
        const hawq_conv_desc &c = st.desc, &e = d.desc;
        const double px = (double)c.H * c.W;     // the last convolution has stride 1: as many input as output pixels
        *macs += d.macs_per_image * N;
        *bytes = (px * c.C + px * e.C + px * c.K) * N + st.bytes_fixed + d.bytes_fixed;
    }
    return HAWQ_OK;
}

// One part of a batch: its images, outputs, workspace and the stream its launches go to
struct Part {
    const void *x;
    int32_t N;
    int32_t *logits;
    uint8_t *ws;
    hipStream_t stream;
    char deferred[256];   // transition steps whose work runs with their block's last convolution
};

// Launch every step for every part, step by step (so that the parts' launches reach their streams interleaved).
// ev (one part only): an event before and after each step.
static hawq_status run_parts(const hawq_net *net, Part *parts, int n_parts, hipEvent_t *ev) {
    if (net->steps.size() > sizeof parts[0].deferred) return HAWQ_ERR_UNSUPPORTED;
    for (size_t s = 0; s < net->steps.size(); ++s)
    for (int pi = 0; pi < n_parts; ++pi) {
        Part &part = parts[pi];
        const void *x = part.x;
        const int32_t N = part.N;
        int32_t *logits = part.logits;
        uint8_t *ws = part.ws;
        hipStream_t stream = part.stream;
        char *deferred = part.deferred;
        auto tptr = [&](int t) -> uint8_t * { return ws + slot_offset(net, net->tensors[t].slot, N); };
        const Step &st = net->steps[s];
        if (ev && hipEventRecord(ev[2 * s], stream) != hipSuccess) return HAWQ_ERR_DEVICE;
        hawq_status rc = HAWQ_OK;
        if (st.kind == STEP_CONV && (st.pair_last >= 0 || (st.pair_ds >= 0 && deferred[st.pair_ds]))) {
            const Step &l = st.pair_last >= 0 ? net->steps[st.pair_last] : st;
            const Step &d = st.pair_last >= 0 ? st : net->steps[st.pair_ds];
            hawq_conv_desc dm = l.desc, dsc = d.desc;
            dm.N = N; dsc.N = N;
            ConvArgs a;
            int x_hi, xs_hi;
            rc = make_dual_args(&dm, tptr(l.in), l.w, l.bias, l.b, l.c, &dsc, tptr(d.in), d.w, d.bias, d.b, d.c, tptr(l.out), true,
                                a, x_hi, xs_hi);
            if (rc != HAWQ_OK) return rc;
            a.mid_s8 = 1; a.res_b = l.res_b; a.res_c = l.res_c;
            a.corun = n_parts > 1;
            a.w_t = l.w_t; a.ws_t = d.w_t;
            a.w_f = l.w_f; a.ws_f = d.w_f;
            a.dual16 = l.dual16;
            if (st.pair_last >= 0) {
                if (pair_runs_fused(net, N, (int)s) && (conv_pws_dual_eligible(a, x_hi, xs_hi) || conv_mfma_dual_eligible(a, x_hi, xs_hi))) {
                    deferred[s] = 1;
                    if (ev && hipEventRecord(ev[2 * s + 1], stream) != hipSuccess) return HAWQ_ERR_DEVICE;
                    continue;
                }
            } else {
                rc = dispatch_conv_dual(a, x_hi, xs_hi, stream);
                if (rc != HAWQ_OK) return rc;
                if (ev && hipEventRecord(ev[2 * s + 1], stream) != hipSuccess) return HAWQ_ERR_DEVICE;
                continue;
            }
        }
        if (st.kind == STEP_CONV && st.tail_next >= 0) {   // runs inside the next step's launch
            if (ev && hipEventRecord(ev[2 * s + 1], stream) != hipSuccess) return HAWQ_ERR_DEVICE;
            continue;
        }
        if (st.kind == STEP_CONV && st.tail_prev >= 0) {
            const Step &p = net->steps[st.tail_prev];
            hawq_conv_desc d2 = p.desc, d3 = st.desc;
            d2.N = N; d3.N = N;
            ConvArgs a1, a2;
            int x_hi, h_hi;
            rc = make_conv_args(&d2, tptr(p.in), p.w, p.bias, p.b, p.c, nullptr, nullptr, nullptr, tptr(st.out), true, a1, x_hi);
            if (rc == HAWQ_OK)
                rc = make_conv_args(&d3, tptr(p.in), st.w, st.bias, st.b, st.c, tptr(st.res), st.res_b, st.res_c, tptr(st.out), true, a2, h_hi);
            if (rc != HAWQ_OK) return rc;
            a1.w_f = p.w_f;
            a1.corun = n_parts > 1;
            RpArgs r;
            if (!make_rp_args(a1, x_hi, &a2, st.w_f, r)) return HAWQ_ERR_UNSUPPORTED;   // (the plan checked shapes and types)
            rc = launch_conv_rp(r, true, stream);
            if (rc != HAWQ_OK) return rc;
            if (ev && hipEventRecord(ev[2 * s + 1], stream) != hipSuccess) return HAWQ_ERR_DEVICE;
            continue;
        }
        const uint8_t *in = st.in >= 0 ? tptr(st.in) : (const uint8_t *)x;
        uint8_t *outp = st.out >= 0 ? tptr(st.out) : (uint8_t *)logits;
        switch (st.kind) {
        case STEP_STEM:
        case STEP_CONV:
        case STEP_FC: {
            hawq_conv_desc d = st.desc;
            if (st.kind == STEP_FC) { d.W = N; } else { d.N = N; }
            ConvArgs a;
            int x_hi;
            const uint8_t *res = st.res >= 0 ? tptr(st.res) : nullptr;
            const bool raw = st.kind == STEP_FC || st.raw;
            rc = make_conv_args(&d, in, st.w, st.bias, raw ? nullptr : st.b, raw ? nullptr : st.c, res, st.res_b, st.res_c,
                                outp, true, a, x_hi);
            a.corun = n_parts > 1;
            a.w_t = st.w_t;
            a.w_f = st.w_f;
            if (rc == HAWQ_OK) {
                if (st.kind == STEP_STEM && st.fused_pool && conv_stem_eligible(a)) {
                    const Step &pool = net->steps[s + 1];
                    a.w = st.w_stem;
                    a.bias = st.bias_stem;
                    rc = launch_conv_stem_pool(a, pool.desc.y_dtype, pool.desc.y_lo, pool.desc.y_hi, tptr(pool.out), stream);
                } else if (st.kind == STEP_STEM && st.fused_pool) {
                    rc = HAWQ_ERR_UNSUPPORTED;   // the image pointer is not 16-byte aligned
                } else if (st.kind == STEP_STEM && conv_stem_eligible(a)) {
                    a.w = st.w_stem;
                    a.bias = st.bias_stem;
                    rc = launch_conv_stem(a, stream);
                } else {
                    rc = dispatch_conv(a, x_hi, stream);
                }
            }
            break;
        }
        case STEP_CONV_DUAL: {
            hawq_conv_desc d = st.desc, dsc = st.desc_s;
            d.N = N; dsc.N = N;
            ConvArgs a;
            int x_hi, xs_hi;
            rc = make_dual_args(&d, in, st.w, st.bias, st.b, st.c, &dsc, tptr(st.res), st.w_s, st.bias_s, st.b_s, st.c_s, outp,
                                true, a, x_hi, xs_hi);
            a.corun = n_parts > 1;
            a.w_t = st.w_t; a.ws_t = st.w_s_t;
            a.w_f = st.w_f; a.ws_f = st.w_s_f;
            a.dual16 = st.dual16;
            if (rc == HAWQ_OK) rc = dispatch_conv_dual(a, x_hi, xs_hi, stream);
            break;
        }
        case STEP_RESADD:
            rc = launch_residual_add((int64_t)N * st.desc.H * st.desc.W, st.desc.K, HAWQ_S32, HAWQ_S32, st.desc.y_dtype, in, st.b,
                                     st.c, tptr(st.res), st.b_s, st.c_s, st.desc.y_lo, st.desc.y_hi, outp, stream);
            break;
        case STEP_MAXPOOL:
            if (st.skip && net->steps[s - 1].fused_pool) break;   // done inside conv1's kernel
            rc = launch_maxpool(N, st.desc.H, st.desc.W, st.desc.C, st.desc.x_dtype, st.desc.y_dtype, in, st.desc.y_lo,
                                st.desc.y_hi, outp, stream);
            break;
        case STEP_AVGPOOL:
            rc = launch_avgpool(N, st.desc.H * st.desc.W, st.desc.C, st.desc.x_dtype, st.desc.y_dtype, in, st.b, st.c,
                                st.desc.y_lo, st.desc.y_hi, outp, stream);
            break;
        }
        if (rc != HAWQ_OK) return rc;
        if (ev && hipEventRecord(ev[2 * s + 1], stream) != hipSuccess) return HAWQ_ERR_DEVICE;
    }
    return HAWQ_OK;
}

static hawq_status run_forward(const hawq_net *net, const void *x, int32_t N, int32_t *logits, void *workspace,
                               size_t workspace_bytes, hipStream_t stream, hipEvent_t *ev) {
    if (!net || !x || !logits || !workspace) return HAWQ_ERR_NULL;
    if (N <= 0) return HAWQ_ERR_SHAPE;
    if (workspace_bytes < hawq_net_workspace_bytes(net, N)) return HAWQ_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 255) return HAWQ_ERR_UNSUPPORTED;
    Part parts[2] = {};
    parts[0].x = x; parts[0].N = N; parts[0].logits = logits; parts[0].ws = (uint8_t *)workspace; parts[0].stream = stream;
    const int n1 = ev ? 0 : split_first_part(net, N);   // (per-step timing: one part, one stream)
    if (n1 <= 0) return run_parts(net, parts, 1, ev);
    // two parts: images [0, n1) on the caller's stream, [n1, N) on the net's second stream, which starts after everything
    // already queued on the caller's stream and which the caller's stream waits for at the end
    const size_t image_bytes = (size_t)net->hw * net->hw * 3;
    parts[0].N = n1;
    parts[1].x = (const uint8_t *)x + (size_t)n1 * image_bytes;
    parts[1].N = N - n1;
    parts[1].logits = logits + (size_t)n1 * net->classes;
    parts[1].ws = (uint8_t *)workspace + workspace_one_part(net, n1);
    parts[1].stream = net->aux_stream;
    if (hipEventRecord(net->fork_ev, stream) != hipSuccess) return HAWQ_ERR_DEVICE;
    if (hipStreamWaitEvent(net->aux_stream, net->fork_ev, 0) != hipSuccess) return HAWQ_ERR_DEVICE;
    const hawq_status rc = run_parts(net, parts, 2, nullptr);
    // join even after a failed launch, so that the caller's stream never runs ahead of work queued on the second one
    if (hipEventRecord(net->join_ev, net->aux_stream) != hipSuccess) return HAWQ_ERR_DEVICE;
    if (hipStreamWaitEvent(stream, net->join_ev, 0) != hipSuccess) return HAWQ_ERR_DEVICE;
    return rc;
}

// Measurement hook (not part of the documented interface): 0 = the library's rule, -1 = never split a batch, n = first part of n images.
// Set it before sizing the workspace.
void hawq_tune_set_split(int32_t n_first) { g_split_override = n_first; }

void hawq_tune_set_fusion(int32_t mode) { g_fuse_tails = mode; }

hawq_status hawq_forward_resnet(const hawq_net *net, const void *x, int32_t N, int32_t *logits, void *workspace,
                                size_t workspace_bytes, void *stream) {
    return run_forward(net, x, N, logits, workspace, workspace_bytes, (hipStream_t)stream, nullptr);
}

size_t hawq_noalloc_workspace_limit(void) { return (size_t)HAWQ_NOALLOC_SCRATCH_BYTES; }

hawq_status hawq_forward_resnet_noalloc(const hawq_net *net, const void *x, int32_t N, int32_t *logits, void *stream) {
    if (!net || !x || !logits) return HAWQ_ERR_NULL;
    if (N <= 0) return HAWQ_ERR_SHAPE;
    if (hawq_net_workspace_bytes(net, N) > (size_t)HAWQ_NOALLOC_SCRATCH_BYTES) return HAWQ_ERR_WORKSPACE;
    void *ws = scratch_base();
    if (ws == nullptr) return HAWQ_ERR_DEVICE;
    return run_forward(net, x, N, logits, ws, (size_t)HAWQ_NOALLOC_SCRATCH_BYTES, (hipStream_t)stream, nullptr);
}

hawq_status hawq_forward_resnet_timed(const hawq_net *net, const void *x, int32_t N, int32_t *logits, void *workspace,
                                      size_t workspace_bytes, void *stream, float *step_ms) {
    if (!net || !step_ms) return HAWQ_ERR_NULL;
    const size_t ns = net->steps.size();
    std::vector<hipEvent_t> ev(2 * ns);
    for (auto &e : ev)
        if (hipEventCreate(&e) != hipSuccess) return HAWQ_ERR_DEVICE;
    hawq_status rc = run_forward(net, x, N, logits, workspace, workspace_bytes, (hipStream_t)stream, ev.data());
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess && rc == HAWQ_OK) rc = HAWQ_ERR_DEVICE;
    if (rc == HAWQ_OK)
        for (size_t s = 0; s < ns; ++s)
            if (hipEventElapsedTime(&step_ms[s], ev[2 * s], ev[2 * s + 1]) != hipSuccess) rc = HAWQ_ERR_DEVICE;
    for (auto &e : ev) (void)hipEventDestroy(e);
    return rc;
}

}  // extern "C"
