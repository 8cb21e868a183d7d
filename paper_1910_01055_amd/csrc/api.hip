// C ABI of the library: the policy handle, argument checks and the launch sequences.
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hpp"

using namespace aq;

// Scratch of aq_policy_forward_int8_static: the intermediate activations of the one-launch-per-layer plan for
// callers that cannot allocate.  The array is part of the library's device image, so every GPU the library
// runs on holds its own copy at its own address until the process ends; host code never uses the array's
// name as an address (it is only a host-side stand-in), but the per-device pointer looked up below.
static __device__ __align__(256) unsigned char scratch[AQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];  // per device, filled on first use with that device current

// device address of `scratch` on the current device (AQ_EHIP when the lookup fails)
aq_status static_scratch(unsigned char** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AQ_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return AQ_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = (unsigned char*)g_scratch_ptr[dev];
    return AQ_OK;
}
}  // namespace

namespace {

struct LayerBuf {
    aq_layer d;
    int K, N, K_pad, N_pad, KS, NT, oh, ow;
    bool fc;
    int8_t* wp;
    float* s_w;
    int32_t* z_w;
    int32_t* rowsum;
    int32_t* bias_q;
    int32_t* M0;
    int32_t* rshift;
    float* m;
    // The constants an epilogue reads per output channel sit in one contiguous pack of four
    // [N_pad] arrays, so that the fused kernel stages them with one linear copy:
    //   [0] bias_fold   [1] M0 (requantized layers) or m (LayerNorm and last layers)
    //   [2] rz or gamma [3] sh or beta          (a layer is either requantized or normalised)
    int32_t* bias_fold;
    int32_t* pack1;
    int32_t* rz;
    int32_t* sh;
    float* gamma;
    float* beta;
};

}  // namespace

struct aq_policy {
    aq_net net;
    std::vector<LayerBuf> L;
    void* slab = nullptr;  // all per-layer buffers live in one allocation
    ActQ* actq = nullptr;
    int* status = nullptr;
    uint32_t* mm = nullptr;
    uint32_t* keys = nullptr;
    NetDev h_net{};            // host copy of the device-resident network description
    NetDev* d_net = nullptr;
    QTab h_qtab{};             // the quantizer's table of the policy, host copy and device copy
    QTab* d_qtab = nullptr;
    bool quantized = false;
    size_t layer_bytes = 0;    // the slab's leading part: every layer's packed weights and constants
    uint64_t net_hash = 0;     // of the network description (blob header)
    int path = 0;  // 0 auto, 1 fused only, 2 one launch per layer, 3 one launch per layer also for the convolutions
    bool conv_stack = true;
    bool subbyte = false;  // plan 4: plan 2 with the few-row layers streaming the nibble copies of their weights
    // activation scratch of the per-layer path (8-bit maps, the fp32 rows a LayerNorm layer hands to its row
    // kernel, the logits of an argmax head) and of the fp32 actor, grown on demand
    int64_t cap_i8 = 0, cap_f32 = 0;
    int8_t* act_i8[2] = {nullptr, nullptr};
    float* ln_x = nullptr;
    float* y_rows = nullptr;
    float* act_f32[2] = {nullptr, nullptr};
    int64_t ln_elems = 0;  // per sample: widest LayerNorm layer output
    int64_t y_elems = 0;   // per sample: logits kept for an argmax head
    // half-precision actor: binary16 weights in operand order and rounded bias / gain / offset per layer
    // (one allocation, made by the first aq_convert_params_fp16), and its activation scratch
    void* h16_slab = nullptr;
    std::vector<void*> h16_wp;
    std::vector<float*> h16_bias, h16_gamma, h16_beta;
    bool h16_ready = false;
    int64_t cap_f16 = 0;
    void* act_f16[2] = {nullptr, nullptr};
    // the learner's fp32 parameters, copied by aq_policy_set_params_fp32 (one allocation at its first call)
    void* f32_slab = nullptr;
    std::vector<float*> f32_w, f32_b, f32_gamma, f32_beta;
    bool f32_ready = false;
    // policies of at most 4 bits, per-channel symmetric, under launch plan 4: the fully connected layers' weights
    // once more as nibbles, for the few-row kernel (one allocation when the plan is first chosen; rewritten by
    // the first forward pass after every quantize / import)
    void* w4_slab = nullptr;
    std::vector<uint8_t*> w4;
    bool w4_stale = true;
    float* calib = nullptr;        // 2 * AQ_MAX_LAYERS floats: (min, max) per activation tensor, for aq_calibrate_fp32
    int64_t max_hidden_elems = 0;  // per sample, over hidden layer outputs
    int64_t max_out_elems = 0;     // per sample, over all layer outputs
};

static void fill_layer_dev(const aq_policy* p, int l, LayerDev& d) {
    const LayerBuf& b = p->L[l];
    d.wp = b.wp;
    d.bias_fold = b.bias_fold;
    d.M0 = b.M0;
    d.rshift = b.rshift;
    d.m = b.m;
    d.gamma = b.gamma;
    d.beta = b.beta;
    d.z_w = b.z_w;
    d.rz = b.rz;
    d.sh = b.sh;
    d.K = b.K;
    d.N = b.N;
    d.KS = b.KS;
    d.NT = b.NT;
    d.act = b.d.act;
    d.in_h = b.d.in_h;
    d.in_w = b.d.in_w;
    d.in_c = b.d.in_c;
    d.kh = b.d.kh;
    d.kw = b.d.kw;
    d.stride = b.d.stride;
    d.oh = b.oh;
    d.ow = b.ow;
}

static hipStream_t as_stream(void* s) { return (hipStream_t)s; }

constexpr int kMaxK = 1 << 16, kMaxN = 1 << 20, kMaxSide = 1 << 14;

extern "C" const char* aq_status_string(aq_status s) {
    switch (s) {
        case AQ_OK: return "ok";
        case AQ_EINVAL: return "invalid argument";
        case AQ_ESHAPE: return "unsupported or inconsistent layer shapes";
        case AQ_ENONFINITE: return "non-finite weights";
        case AQ_ENOTQUANT: return "policy not quantized yet";
        case AQ_EHIP: return "HIP runtime error";
        case AQ_ENOMEM: return "out of device memory";
        case AQ_ERANGE: return "requantization multiplier out of range";
        case AQ_ETOOBIG: return "needs more scratch memory than is available without allocating";
    }
    return "unknown";
}

extern "C" aq_status aq_policy_create(const aq_net* net, aq_policy** out) {
    if (!net || !out || !net->layers) return AQ_EINVAL;
    if (net->n_layers < 1 || net->n_layers > AQ_MAX_LAYERS) return AQ_EINVAL;
    if (net->head < 0 || net->head > AQ_HEAD_LINEAR) return AQ_EINVAL;
    if (net->wscheme != AQ_W_TENSOR_ASYM_U8 && net->wscheme != AQ_W_CHANNEL_SYM_S8) return AQ_EINVAL;
    if (net->in_type != AQ_IN_F32 && net->in_type != AQ_IN_U8) return AQ_EINVAL;
    if (net->qdenom != 255 && net->qdenom != 256) return AQ_EINVAL;
    if (!(net->ln_eps > 0.0f)) return AQ_EINVAL;
    if (net->wbits != 0 && (net->wbits < 2 || net->wbits > 8)) return AQ_EINVAL;
    int dev_count = 0;
    if (hipGetDeviceCount(&dev_count) != hipSuccess || dev_count < 1) return AQ_EHIP;

    aq_policy* p = new (std::nothrow) aq_policy();
    if (!p) return AQ_ENOMEM;
    p->net = *net;
    p->net.layers = nullptr;
    int64_t prev_elems = -1;
    int prev_h = 0, prev_w = 0, prev_c = 0;
    bool prev_conv = false;
    size_t bytes = 0;
    auto take = [&](size_t n) {
        size_t off = bytes;
        bytes += (n + 255) / 256 * 256;
        return off;
    };
    std::vector<size_t> offs;
    for (int l = 0; l < net->n_layers; ++l) {
        const aq_layer& d = net->layers[l];
        LayerBuf b{};
        b.d = d;
        if (d.act < 0 || d.act > AQ_ACT_LN_TANH || d.out_c < 1 || d.in_c < 1) {
            delete p;
            return AQ_EINVAL;
        }
        // Size limits: K products of two signed 8-bit values (each at most 2^14 in magnitude) must stay
        // inside the int32 accumulator, and tile counts and per-sample element counts inside int32.
        if (d.in_c > kMaxK || d.out_c > kMaxN ||
            (d.kind == AQ_CONV2D && (d.in_h > kMaxSide || d.in_w > kMaxSide ||
                                     (int64_t)d.kh * d.kw * d.in_c > kMaxK))) {
            delete p;
            return AQ_ESHAPE;
        }
        if (d.kind == AQ_FC) {
            b.fc = true;
            b.K = d.in_c;
            b.oh = b.ow = 1;
            b.d.in_h = b.d.in_w = b.d.kh = b.d.kw = b.d.stride = 1;
            if (prev_elems >= 0 && prev_elems != d.in_c) {
                delete p;
                return AQ_ESHAPE;
            }
        } else if (d.kind == AQ_CONV2D) {
            b.fc = false;
            if (d.kh < 1 || d.kw < 1 || d.stride < 1 || d.in_h < d.kh || d.in_w < d.kw) {
                delete p;
                return AQ_ESHAPE;
            }
            if (l > 0 && (!prev_conv || prev_h != d.in_h || prev_w != d.in_w || prev_c != d.in_c)) {
                delete p;
                return AQ_ESHAPE;
            }
            if (d.act == AQ_ACT_LN_TANH) {
                delete p;
                return AQ_ESHAPE;
            }
            b.K = d.kh * d.kw * d.in_c;
            b.oh = (d.in_h - d.kh) / d.stride + 1;
            b.ow = (d.in_w - d.kw) / d.stride + 1;
        } else {
            delete p;
            return AQ_EINVAL;
        }
        b.N = d.out_c;
        b.K_pad = round_up(b.K, kTile);
        b.N_pad = round_up(b.N, kTile);
        b.KS = b.K_pad / kTile;
        b.NT = b.N_pad / kTile;
        prev_conv = !b.fc;
        prev_h = b.oh;
        prev_w = b.ow;
        prev_c = b.N;
        prev_elems = (int64_t)b.oh * b.ow * b.N;
        if (l < net->n_layers - 1 && prev_elems > p->max_hidden_elems) p->max_hidden_elems = prev_elems;
        if (prev_elems > p->max_out_elems) p->max_out_elems = prev_elems;
        if (l < net->n_layers - 1 && d.act == AQ_ACT_LN_TANH && prev_elems > p->ln_elems) p->ln_elems = prev_elems;
        if (l == net->n_layers - 1 && net->head == AQ_HEAD_ARGMAX) p->y_elems = prev_elems;
        offs.push_back(take((size_t)b.NT * b.KS * 1024));
        for (int i = 0; i < 7; ++i) offs.push_back(take((size_t)b.N_pad * 4));
        offs.push_back(take((size_t)b.N_pad * 4 * 4));  // the epilogue constant pack, see LayerBuf
        p->L.push_back(b);
    }
    p->layer_bytes = bytes;
    size_t off_status = take(256);
    size_t off_mm = take(256);
    size_t off_keys = take(sizeof(uint32_t) * 2 * (AQ_MAX_LAYERS + 1));
    size_t off_net = take(sizeof(NetDev));
    size_t off_qtab = take(sizeof(QTab));
    size_t off_calib = take(sizeof(float) * 2 * AQ_MAX_LAYERS);
    if (hipMalloc(&p->slab, bytes) != hipSuccess) {
        delete p;
        return AQ_ENOMEM;
    }
    // zero once: padding rows / k-steps of the packed weights and padded constants stay zero for good
    if (hipMemset(p->slab, 0, bytes) != hipSuccess) {
        (void)hipFree(p->slab);
        delete p;
        return AQ_EHIP;
    }
    p->w4.assign(p->L.size(), nullptr);
    char* base = (char*)p->slab;
    size_t oi = 0;
    for (auto& b : p->L) {
        b.wp = (int8_t*)(base + offs[oi++]);
        b.s_w = (float*)(base + offs[oi++]);
        b.z_w = (int32_t*)(base + offs[oi++]);
        b.rowsum = (int32_t*)(base + offs[oi++]);
        b.bias_q = (int32_t*)(base + offs[oi++]);
        b.M0 = (int32_t*)(base + offs[oi++]);
        b.rshift = (int32_t*)(base + offs[oi++]);
        b.m = (float*)(base + offs[oi++]);
        int32_t* pack = (int32_t*)(base + offs[oi++]);
        b.bias_fold = pack;
        b.pack1 = pack + b.N_pad;
        b.rz = pack + 2 * b.N_pad;
        b.sh = pack + 3 * b.N_pad;
        b.gamma = (float*)b.rz;
        b.beta = (float*)b.sh;
    }
    p->status = (int*)(base + off_status);
    p->mm = (uint32_t*)(base + off_mm);
    p->keys = (uint32_t*)(base + off_keys);
    p->d_net = (NetDev*)(base + off_net);
    p->d_qtab = (QTab*)(base + off_qtab);
    p->calib = (float*)(base + off_calib);
    p->actq = p->d_net->actq;  // device address arithmetic only
    for (int l = 0; l < net->n_layers; ++l) {
        fill_layer_dev(p, l, p->h_net.L[l]);
    }
    p->h_net.n_layers = net->n_layers;
    p->h_net.head = net->head;
    p->h_net.in_u8 = net->in_type == AQ_IN_U8;
    p->h_net.asym = net->wscheme == AQ_W_TENSOR_ASYM_U8;
    p->h_net.ln_eps = net->ln_eps;
    {   // the quantizer's table: outputs per layer and each layer's first workgroup in the shared grids
        QTab& q = p->h_qtab;
        q.n_layers = net->n_layers;
        q.asym = p->h_net.asym;
        q.in_u8 = p->h_net.in_u8;
        q.qdenom = (float)net->qdenom;
        const int wbits = net->wbits ? net->wbits : 8;
        q.w_qmax = (1 << wbits) - 1;
        q.w_qw = (1 << (wbits - 1)) - 1;
        q.w_qdenom = net->qdenom == 256 ? (float)(q.w_qmax + 1) : (float)q.w_qmax;
        int row_blk = 0, cst_blk = 0, rng_blk = 0;
        for (int l = 0; l < net->n_layers; ++l) {
            const LayerBuf& b = p->L[l];
            QLayerTab& t = q.L[l];
            t.wp = b.wp; t.s_w = b.s_w; t.z_w = b.z_w; t.rowsum = b.rowsum; t.bias_q = b.bias_q; t.M0 = b.M0;
            t.rshift = b.rshift; t.m = b.m; t.bias_fold = b.bias_fold; t.pack1 = b.pack1; t.rz = b.rz; t.sh = b.sh;
            t.N = b.N; t.K = b.K; t.KS = b.KS;
            t.ln = b.d.act == AQ_ACT_LN_TANH;
            t.requant = l < net->n_layers - 1 && !t.ln;
            t.row_blk0 = row_blk;
            t.cst_blk0 = cst_blk;
            t.rng_blk0 = rng_blk;
            const int64_t n4 = (int64_t)b.N * b.K / 4 + 1;
            int64_t rb = (n4 + 255) / 256;
            t.rng_blks = (int)(rb < 1 ? 1 : (rb > 256 ? 256 : rb));
            row_blk += (b.N + 3) / 4;
            cst_blk += (b.N + 255) / 256;
            rng_blk += t.rng_blks;
        }
        q.row_blks = row_blk;
        q.cst_blks = cst_blk;
        q.rng_blks_total = rng_blk;
        if (hipMemcpy(p->d_qtab, &q, sizeof(QTab), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(p->slab);
            delete p;
            return AQ_EHIP;
        }
    }
    {   // FNV-1a over everything that fixes the blob's layout and meaning
        uint64_t h = 1469598103934665603ull;
        auto mix = [&](int64_t v) {
            for (int i = 0; i < 8; ++i) {
                h ^= (uint64_t)(v >> (8 * i)) & 0xffu;
                h *= 1099511628211ull;
            }
        };
        mix(net->n_layers);
        mix(net->head);
        mix(net->wscheme);
        mix(net->in_type);
        mix(net->qdenom);
        mix(net->wbits ? net->wbits : 8);
        for (const auto& b : p->L) {
            mix(b.d.kind); mix(b.d.in_h); mix(b.d.in_w); mix(b.d.in_c); mix(b.d.out_c);
            mix(b.d.kh); mix(b.d.kw); mix(b.d.stride); mix(b.d.act);
        }
        mix((int64_t)p->layer_bytes);
        p->net_hash = h;
    }
    if (hipMemcpy(p->d_net, &p->h_net, sizeof(NetDev), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(p->slab);
        delete p;
        return AQ_EHIP;
    }
    {   // set-up of the allocation-free forward: this device's address of the static scratch
        unsigned char* sc = nullptr;
        if (static_scratch(&sc) != AQ_OK) {
            (void)hipFree(p->slab);
            delete p;
            return AQ_EHIP;
        }
    }
    *out = p;
    return AQ_OK;
}

extern "C" aq_status aq_policy_destroy(aq_policy* p) {
    if (!p) return AQ_EINVAL;
    (void)hipDeviceSynchronize();
    if (p->slab) (void)hipFree(p->slab);
    if (p->w4_slab) (void)hipFree(p->w4_slab);
    for (int i = 0; i < 2; ++i) {
        if (p->act_i8[i]) (void)hipFree(p->act_i8[i]);
        if (p->act_f32[i]) (void)hipFree(p->act_f32[i]);
        if (p->act_f16[i]) (void)hipFree(p->act_f16[i]);
    }
    if (p->ln_x) (void)hipFree(p->ln_x);
    if (p->y_rows) (void)hipFree(p->y_rows);
    if (p->h16_slab) (void)hipFree(p->h16_slab);
    if (p->f32_slab) (void)hipFree(p->f32_slab);
    delete p;
    return AQ_OK;
}

// Growing a buffer frees and allocates device memory and waits for the device: not possible while the
// caller's stream is being captured into a graph, which the forward then reports instead of breaking the capture.
static bool capturing(hipStream_t st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone;
}

// bytes of one 8-bit activation map of the per-layer plan (a little slack behind the last row)
static size_t i8_map_bytes(const aq_policy* p, int64_t batch) {
    return (size_t)batch * (size_t)(p->max_hidden_elems > 0 ? p->max_hidden_elems : 1) + 64;
}

static aq_status ensure_i8(aq_policy* p, int64_t batch, hipStream_t st) {
    if (batch <= p->cap_i8) return AQ_OK;
    if (capturing(st)) return AQ_ETOOBIG;
    (void)hipDeviceSynchronize();
    for (int i = 0; i < 2; ++i) {
        if (p->act_i8[i]) (void)hipFree(p->act_i8[i]);
        p->act_i8[i] = nullptr;
    }
    if (p->ln_x) (void)hipFree(p->ln_x);
    if (p->y_rows) (void)hipFree(p->y_rows);
    p->ln_x = p->y_rows = nullptr;
    p->cap_i8 = 0;
    for (int i = 0; i < 2; ++i)
        if (hipMalloc((void**)&p->act_i8[i], i8_map_bytes(p, batch)) != hipSuccess) return AQ_ENOMEM;
    // fp32 rows exist only where the 8-bit path needs them: LayerNorm inputs, argmax logits
    if (p->ln_elems && hipMalloc((void**)&p->ln_x, (size_t)batch * p->ln_elems * 4 + 256) != hipSuccess) return AQ_ENOMEM;
    if (p->y_elems && hipMalloc((void**)&p->y_rows, (size_t)batch * p->y_elems * 4 + 256) != hipSuccess) return AQ_ENOMEM;
    p->cap_i8 = batch;
    return AQ_OK;
}

static aq_status ensure_f32(aq_policy* p, int64_t batch, hipStream_t st) {
    if (batch <= p->cap_f32) return AQ_OK;
    if (capturing(st)) return AQ_ETOOBIG;
    (void)hipDeviceSynchronize();
    for (int i = 0; i < 2; ++i) {
        if (p->act_f32[i]) (void)hipFree(p->act_f32[i]);
        p->act_f32[i] = nullptr;
    }
    p->cap_f32 = 0;
    size_t n = ((size_t)batch * (size_t)p->max_out_elems + 64) * sizeof(float);
    for (int i = 0; i < 2; ++i)
        if (hipMalloc((void**)&p->act_f32[i], n) != hipSuccess) return AQ_ENOMEM;
    p->cap_f32 = batch;
    return AQ_OK;
}

static aq_status ensure_f16(aq_policy* p, int64_t batch, hipStream_t st) {
    if (batch <= p->cap_f16) return AQ_OK;
    if (capturing(st)) return AQ_ETOOBIG;
    (void)hipDeviceSynchronize();
    for (int i = 0; i < 2; ++i) {
        if (p->act_f16[i]) (void)hipFree(p->act_f16[i]);
        p->act_f16[i] = nullptr;
    }
    p->cap_f16 = 0;
    size_t n = ((size_t)batch * (size_t)p->max_out_elems + 64) * 2;
    for (int i = 0; i < 2; ++i)
        if (hipMalloc(&p->act_f16[i], n) != hipSuccess) return AQ_ENOMEM;
    p->cap_f16 = batch;
    return AQ_OK;
}

extern "C" aq_status aq_policy_reserve(aq_policy* p, int64_t max_batch) {
    if (!p || max_batch < 0) return AQ_EINVAL;
    aq_status s = ensure_i8(p, max_batch, nullptr);
    if (s != AQ_OK) return s;
    if (p->h16_ready) {
        s = ensure_f16(p, max_batch, nullptr);
        if (s != AQ_OK) return s;
    }
    return ensure_f32(p, max_batch, nullptr);
}

extern "C" aq_status aq_policy_set_path(aq_policy* p, int32_t path) {
    if (!p || path < 0 || path > 4) return AQ_EINVAL;
    if (path == 4 && !p->w4_slab && p->net.wbits != 0 && p->net.wbits <= 4 && p->net.wscheme == AQ_W_CHANNEL_SYM_S8) {
        size_t w4_bytes = 0;
        std::vector<size_t> need(p->L.size(), 0);
        for (size_t l = 0; l < p->L.size(); ++l) {
            const LayerBuf& b = p->L[l];
            LayerDev probe{};
            probe.kh = probe.kw = probe.in_h = probe.in_w = b.fc ? 1 : 2;
            probe.KS = b.KS;
            if (skinny_layer_supported(probe, 1)) need[l] = (size_t)b.NT * b.KS * 512;
            w4_bytes += need[l];
        }
        if (w4_bytes) {
            if (hipMalloc(&p->w4_slab, w4_bytes) != hipSuccess) return AQ_ENOMEM;
            size_t o4 = 0;
            for (size_t l = 0; l < p->L.size(); ++l) {
                if (!need[l]) continue;
                p->w4[l] = (uint8_t*)p->w4_slab + o4;
                o4 += need[l];
            }
            p->w4_stale = true;
        }
    }
    p->conv_stack = path != 3;
    p->subbyte = path == 4;
    p->path = path >= 3 ? 2 : path;
    return AQ_OK;
}

extern "C" aq_status aq_policy_conv_stack_layers(const aq_policy* p, int32_t* n_layers) {
    if (!p || !n_layers) return AQ_EINVAL;
    FwdArgs a{};
    a.net = p->h_net;
    a.c.batch = 1;
    *n_layers = p->conv_stack ? conv_stack_layers(a) : 0;
    return AQ_OK;
}

extern "C" aq_status aq_policy_fused_plan(const aq_policy* p, int64_t batch, int32_t* rows, int32_t* tiles,
                                          int32_t* kind) {
    if (!p || !rows || !tiles || !kind || batch < 1) return AQ_EINVAL;
    FwdArgs a{};
    a.net = p->h_net;
    a.c.batch = batch;
    int r = 0, t = 0;
    size_t lds = 0;
    if (p->path == 2 || !fused_mlp_supported(a, &r, &lds, &t)) r = t = 0;
    *rows = r;
    *tiles = t;
    *kind = r != 0 ? fused_mlp_kernel_kind(a) : 0;
    return AQ_OK;
}

extern "C" aq_status aq_policy_subbyte_layers(const aq_policy* p, int64_t batch, int32_t* n_layers) {
    if (!p || !n_layers || batch < 1) return AQ_EINVAL;
    FwdArgs a{};
    a.net = p->h_net;
    a.c.batch = batch;
    int r = 0;
    size_t lds = 0;
    int n = 0;
    if (p->path == 2 || !fused_mlp_supported(a, &r, &lds)) {
        const int nc = p->conv_stack ? conv_stack_layers(a) : 0;
        for (int l = nc; l < (int)p->L.size(); ++l)
            n += p->subbyte && p->w4[l] && !p->h_net.asym && layer_uses_skinny(a, l);
    }
    *n_layers = n;
    return AQ_OK;
}

extern "C" aq_status aq_policy_status(aq_policy* p, void* stream) {
    if (!p) return AQ_EINVAL;
    int h2[2] = {0, 0};  // [0] the 8-bit policy's status word, [1] the half-precision policy's
    AQ_HIP_CHECK(hipStreamSynchronize(as_stream(stream)));
    AQ_HIP_CHECK(hipMemcpy(h2, p->status, sizeof(h2), hipMemcpyDeviceToHost));
    const int h = h2[0] | (h2[1] & kStatNonFinite);
    if (h & kStatNonFinite) return AQ_ENONFINITE;
    if (h & kStatRange) return AQ_ERANGE;
    if (h & kStatBlob) return AQ_EINVAL;
    return AQ_OK;
}

// ---- policy blob: [64-byte header][128-byte tail: activation (scale, zero-point) pairs and
// short-form flags][the slab's layer part]
namespace {
constexpr size_t kBlobHeader = 64, kBlobTail = 128;
constexpr uint32_t kBlobMagic = 0x42515141u;  // "AQQB"
constexpr uint32_t kBlobVersion = 1;
static_assert(sizeof(ActQ) * (AQ_MAX_LAYERS + 1) + sizeof(int) * AQ_MAX_LAYERS <= kBlobTail, "tail fits");
static_assert(offsetof(NetDev, fast) == offsetof(NetDev, actq) + sizeof(ActQ) * (AQ_MAX_LAYERS + 1),
              "scales, zero-points and flags are contiguous");
void blob_words(const aq_policy* p, uint32_t (&w)[6]) {
    const uint64_t payload = kBlobTail + p->layer_bytes;
    w[0] = kBlobMagic;
    w[1] = kBlobVersion;
    w[2] = (uint32_t)p->net_hash;
    w[3] = (uint32_t)(p->net_hash >> 32);
    w[4] = (uint32_t)payload;
    w[5] = (uint32_t)(payload >> 32);
}
constexpr size_t kTailBytes = sizeof(ActQ) * (AQ_MAX_LAYERS + 1) + sizeof(int) * AQ_MAX_LAYERS;
}  // namespace

// the nibble copies of the weights follow every change of the packed 8-bit operands: written by the first forward
// pass under launch plan 4 after such a change
static aq_status refresh_w4(aq_policy* p, hipStream_t st) {
    for (size_t l = 0; l < p->L.size(); ++l) {
        if (!p->w4[l]) continue;
        const LayerBuf& b = p->L[l];
        const aq_status s = launch_pack_nibbles(b.wp, p->w4[l], (int64_t)b.NT * b.KS * 64, st);
        if (s != AQ_OK) return s;
    }
    p->w4_stale = false;
    return AQ_OK;
}

extern "C" aq_status aq_policy_blob_size(const aq_policy* p, uint64_t* bytes) {
    if (!p || !bytes) return AQ_EINVAL;
    *bytes = kBlobHeader + kBlobTail + p->layer_bytes;
    return AQ_OK;
}

extern "C" aq_status aq_policy_export_blob(const aq_policy* p, void* d_blob, uint64_t bytes, void* stream) {
    if (!p || !d_blob || ((uintptr_t)d_blob & 15)) return AQ_EINVAL;
    if (bytes < kBlobHeader + kBlobTail + p->layer_bytes) return AQ_EINVAL;
    if (!p->quantized) return AQ_ENOTQUANT;
    hipStream_t st = as_stream(stream);
    uint32_t w[6];
    blob_words(p, w);
    char* dst = (char*)d_blob;
    aq_status s = launch_blob_header_write((uint32_t*)dst, w, st);
    if (s != AQ_OK) return s;
    AQ_HIP_CHECK(hipMemcpyAsync(dst + kBlobHeader, p->d_net->actq, kTailBytes, hipMemcpyDeviceToDevice, st));
    AQ_HIP_CHECK(hipMemcpyAsync(dst + kBlobHeader + kBlobTail, p->slab, p->layer_bytes, hipMemcpyDeviceToDevice, st));
    return AQ_OK;
}

extern "C" aq_status aq_policy_import_blob(aq_policy* p, const void* d_blob, uint64_t bytes, void* stream) {
    if (!p || !d_blob || ((uintptr_t)d_blob & 15)) return AQ_EINVAL;
    if (bytes < kBlobHeader + kBlobTail + p->layer_bytes) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    uint32_t w[6];
    blob_words(p, w);
    const char* src = (const char*)d_blob;
    aq_status s = launch_fill_u32((uint32_t*)p->status, 1, 0u, st);
    if (s != AQ_OK) return s;
    s = launch_blob_header_check((const uint32_t*)src, w, p->status, st);
    if (s != AQ_OK) return s;
    AQ_HIP_CHECK(hipMemcpyAsync(p->d_net->actq, src + kBlobHeader, kTailBytes, hipMemcpyDeviceToDevice, st));
    AQ_HIP_CHECK(hipMemcpyAsync(p->slab, src + kBlobHeader + kBlobTail, p->layer_bytes, hipMemcpyDeviceToDevice, st));
    p->w4_stale = true;
    p->quantized = true;
    return AQ_OK;
}

// ---- packed policy blob: the same header (other magic) and tail, then per layer the weight codes as
// n-bit fields (n = the policy's weight precision) followed by the layer's constants verbatim.
namespace {
constexpr uint32_t kPackedMagic = 0x50515141u;  // "AQQP"
struct PackedLayout {
    std::vector<size_t> w_off, w_bytes, c_off, c_src, c_bytes;  // blob offsets / slab offsets per layer
    size_t total = 0;
};
int policy_wbits(const aq_policy* p) { return p->net.wbits ? p->net.wbits : 8; }
PackedLayout packed_layout(const aq_policy* p) {
    PackedLayout L;
    const int bits = policy_wbits(p);
    size_t at = kBlobHeader + kBlobTail;
    const char* base = (const char*)p->slab;
    for (size_t l = 0; l < p->L.size(); ++l) {
        const LayerBuf& b = p->L[l];
        const size_t wb = (size_t)b.NT * b.KS * 1024;
        const size_t begin = (size_t)((const char*)b.wp - base);
        const size_t end = l + 1 < p->L.size() ? (size_t)((const char*)p->L[l + 1].wp - base) : p->layer_bytes;
        L.w_off.push_back(at);
        L.w_bytes.push_back(wb / 8 * bits);
        at += (wb / 8 * bits + 255) / 256 * 256;
        L.c_off.push_back(at);
        L.c_src.push_back(begin + wb);
        L.c_bytes.push_back(end - begin - wb);
        at += end - begin - wb;
    }
    L.total = at;
    return L;
}
void packed_words(const aq_policy* p, const PackedLayout& L, uint32_t (&w)[6]) {
    blob_words(p, w);
    w[0] = kPackedMagic;
    w[4] = (uint32_t)(L.total - kBlobHeader);
    w[5] = (uint32_t)((uint64_t)(L.total - kBlobHeader) >> 32);
}
}  // namespace

extern "C" aq_status aq_policy_packed_blob_size(const aq_policy* p, uint64_t* bytes) {
    if (!p || !bytes) return AQ_EINVAL;
    *bytes = packed_layout(p).total;
    return AQ_OK;
}

extern "C" aq_status aq_policy_export_packed_blob(const aq_policy* p, void* d_blob, uint64_t bytes, void* stream) {
    if (!p || !d_blob || ((uintptr_t)d_blob & 15)) return AQ_EINVAL;
    const PackedLayout L = packed_layout(p);
    if (bytes < L.total) return AQ_EINVAL;
    if (!p->quantized) return AQ_ENOTQUANT;
    hipStream_t st = as_stream(stream);
    uint32_t w[6];
    packed_words(p, L, w);
    char* dst = (char*)d_blob;
    aq_status s = launch_blob_header_write((uint32_t*)dst, w, st);
    if (s != AQ_OK) return s;
    AQ_HIP_CHECK(hipMemcpyAsync(dst + kBlobHeader, p->d_net->actq, kTailBytes, hipMemcpyDeviceToDevice, st));
    const int bits = policy_wbits(p);
    const int off = p->h_net.asym ? 128 : (1 << (bits - 1)) - 1;
    for (size_t l = 0; l < p->L.size(); ++l) {
        const LayerBuf& b = p->L[l];
        s = launch_pack_bits(b.wp, (uint8_t*)dst + L.w_off[l], (int64_t)b.NT * b.KS * 1024, bits, off, st);
        if (s != AQ_OK) return s;
        const size_t gap = L.c_off[l] - (L.w_off[l] + L.w_bytes[l]);  // alignment padding: a multiple of 4, kept zero
        if (gap) {
            s = launch_fill_u32((uint32_t*)(dst + L.w_off[l] + L.w_bytes[l]), (int)(gap / 4), 0u, st);
            if (s != AQ_OK) return s;
        }
        AQ_HIP_CHECK(hipMemcpyAsync(dst + L.c_off[l], (const char*)p->slab + L.c_src[l], L.c_bytes[l],
                                    hipMemcpyDeviceToDevice, st));
    }
    return AQ_OK;
}

extern "C" aq_status aq_policy_import_packed_blob(aq_policy* p, const void* d_blob, uint64_t bytes, void* stream) {
    if (!p || !d_blob || ((uintptr_t)d_blob & 15)) return AQ_EINVAL;
    const PackedLayout L = packed_layout(p);
    if (bytes < L.total) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    uint32_t w[6];
    packed_words(p, L, w);
    const char* src = (const char*)d_blob;
    aq_status s = launch_fill_u32((uint32_t*)p->status, 1, 0u, st);
    if (s != AQ_OK) return s;
    s = launch_blob_header_check((const uint32_t*)src, w, p->status, st);
    if (s != AQ_OK) return s;
    AQ_HIP_CHECK(hipMemcpyAsync(p->d_net->actq, src + kBlobHeader, kTailBytes, hipMemcpyDeviceToDevice, st));
    const int bits = policy_wbits(p);
    const int off = p->h_net.asym ? 128 : (1 << (bits - 1)) - 1;
    for (size_t l = 0; l < p->L.size(); ++l) {
        const LayerBuf& b = p->L[l];
        s = launch_unpack_bits((const uint8_t*)src + L.w_off[l], b.wp, (int64_t)b.NT * b.KS * 1024, bits, off, b.N, b.K,
                               b.KS, st);
        if (s != AQ_OK) return s;
        AQ_HIP_CHECK(hipMemcpyAsync((char*)p->slab + L.c_src[l], src + L.c_off[l], L.c_bytes[l],
                                    hipMemcpyDeviceToDevice, st));
    }
    p->w4_stale = true;
    p->quantized = true;
    return AQ_OK;
}

static aq_status explore_args_ok(const aq_policy* p, const aq_explore* ex, int64_t batch) {
    if (batch > 0xffffffffLL) return AQ_EINVAL;
    const bool discrete = p->net.head == AQ_HEAD_ARGMAX;
    if (!discrete && !ex->d_sigma) return AQ_EINVAL;
    if (discrete && !(ex->epsilon >= 0.0f && ex->epsilon <= 1.0f)) return AQ_EINVAL;
    return AQ_OK;
}

extern "C" aq_status aq_policy_explore(const aq_policy* p, void* d_actions, int64_t batch, const aq_explore* ex,
                                       void* stream) {
    if (!p || !d_actions || !ex || batch < 0) return AQ_EINVAL;
    const aq_status es = explore_args_ok(p, ex, batch);
    if (es != AQ_OK) return es;
    if (batch == 0) return AQ_OK;
    const int A = p->L.back().N * p->L.back().oh * p->L.back().ow;
    return launch_explore(d_actions, batch, A, p->net.head, ex->d_sigma, ex->epsilon, ex->seed, ex->step,
                          as_stream(stream));
}

extern "C" aq_status aq_quantize_tensor(const float* d_w, int64_t rows, int64_t cols, int32_t wscheme,
                                        int32_t qdenom, void* d_codes, float* d_scale, int32_t* d_zp,
                                        void* d_workspace, void* stream) {
    if (!d_w || !d_codes || !d_scale || !d_zp || !d_workspace) return AQ_EINVAL;
    if (rows < 0 || cols < 0) return AQ_EINVAL;
    // qdenom = 2^n - 1 (default reading) or 2^n (literal) for n = 2..8 bits
    int bits = 0;
    for (int n = 2; n <= 8; ++n)
        if (qdenom == (1 << n) - 1 || qdenom == (1 << n)) bits = n;
    if (bits == 0) return AQ_EINVAL;
    if (wscheme != AQ_W_TENSOR_ASYM_U8 && wscheme != AQ_W_CHANNEL_SYM_S8) return AQ_EINVAL;
    if (cols % 4 != 0 || ((uintptr_t)d_w & 15) || ((uintptr_t)d_codes & 3)) return AQ_ESHAPE;
    if (rows > 0x7fffffffLL || cols / 4 > 0x7fffffffLL) return AQ_ESHAPE;
    if (rows == 0 || cols == 0) return AQ_OK;
    return launch_quantize_tensor(d_w, rows, cols, wscheme, (float)qdenom, (1 << bits) - 1, (1 << (bits - 1)) - 1,
                                  d_codes, d_scale, d_zp, (uint32_t*)d_workspace, as_stream(stream));
}

extern "C" aq_status aq_stream_reference(const float* d_in, int64_t n, void* d_out, void* stream) {
    if (!d_in || !d_out || n < 0) return AQ_EINVAL;
    if (n % 4 != 0 || ((uintptr_t)d_in & 15) || ((uintptr_t)d_out & 3)) return AQ_ESHAPE;
    if (n == 0) return AQ_OK;
    return launch_stream_reference(d_in, n, d_out, as_stream(stream));
}

extern "C" aq_status aq_mfma_loop_reference(const void* d_weights, const void* d_acts, int32_t ksteps, int32_t stream_weights,
                                             int32_t workgroups, int32_t* d_acc, void* stream) {
    if (!d_weights || !d_acts || !d_acc) return AQ_EINVAL;
    if (ksteps < 4 || ksteps % 4 != 0 || workgroups < 1 || workgroups > 65536) return AQ_EINVAL;
    if (((uintptr_t)d_weights & 15) || ((uintptr_t)d_acts & 15) || ((uintptr_t)d_acc & 3)) return AQ_ESHAPE;
    return launch_mfma_reference(d_weights, d_acts, ksteps, stream_weights != 0, workgroups, d_acc, as_stream(stream));
}

extern "C" aq_status aq_quantize_params(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                        const float* const* h_d_gamma, const float* const* h_d_beta,
                                        const aq_range* h_ranges, void* stream) {
    if (!p || !h_ranges) return AQ_EINVAL;
    const int nl = p->net.n_layers;
    if (!h_d_w) {  // the parameters kept by aq_policy_set_params_fp32
        if (h_d_b || h_d_gamma || h_d_beta) return AQ_EINVAL;
        if (!p->f32_ready) return AQ_ENOTQUANT;
        h_d_w = p->f32_w.data();
        h_d_b = p->f32_b.data();
        h_d_gamma = p->f32_gamma.data();
        h_d_beta = p->f32_beta.data();
    }
    for (int l = 0; l < nl; ++l)
        if (!h_d_w[l]) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    RangesArg r{};
    QPtrs ptrs{};
    for (int l = 0; l < nl; ++l) {
        r.lo[l] = h_ranges[l].lo;
        r.hi[l] = h_ranges[l].hi;
        ptrs.w[l] = h_d_w[l];
        ptrs.b[l] = h_d_b ? h_d_b[l] : nullptr;
        ptrs.gamma[l] = h_d_gamma ? h_d_gamma[l] : nullptr;
        ptrs.beta[l] = h_d_beta ? h_d_beta[l] : nullptr;
    }
    aq_status s = launch_quantize_policy(p->d_qtab, p->h_qtab, ptrs, r, p->actq, p->d_net->fast, p->status,
                                         p->mm, st);
    if (s != AQ_OK) return s;
    p->w4_stale = true;
    p->quantized = true;
    return AQ_OK;
}

extern "C" aq_status aq_policy_export_layer(const aq_policy* p, int32_t layer, void* d_codes, float* d_w_scale,
                                            int32_t* d_w_zp, int32_t* d_bias_q, int32_t* d_mult, int32_t* d_rshift,
                                            float* d_m, void* stream) {
    if (!p || layer < 0 || layer >= p->net.n_layers) return AQ_EINVAL;
    if (!p->quantized) return AQ_ENOTQUANT;
    hipStream_t st = as_stream(stream);
    const LayerBuf& b = p->L[layer];
    if (d_codes) {
        aq_status s = launch_unpack_weights(b.wp, b.N, b.K, b.KS, p->net.wscheme == AQ_W_TENSOR_ASYM_U8,
                                            (uint8_t*)d_codes, st);
        if (s != AQ_OK) return s;
    }
    const size_t nb = sizeof(float) * b.N;
    if (d_w_scale) AQ_HIP_CHECK(hipMemcpyAsync(d_w_scale, b.s_w, nb, hipMemcpyDeviceToDevice, st));
    if (d_w_zp) AQ_HIP_CHECK(hipMemcpyAsync(d_w_zp, b.z_w, nb, hipMemcpyDeviceToDevice, st));
    if (d_bias_q) AQ_HIP_CHECK(hipMemcpyAsync(d_bias_q, b.bias_q, nb, hipMemcpyDeviceToDevice, st));
    if (d_mult) AQ_HIP_CHECK(hipMemcpyAsync(d_mult, b.M0, nb, hipMemcpyDeviceToDevice, st));
    if (d_rshift) AQ_HIP_CHECK(hipMemcpyAsync(d_rshift, b.rshift, nb, hipMemcpyDeviceToDevice, st));
    if (d_m) AQ_HIP_CHECK(hipMemcpyAsync(d_m, b.m, nb, hipMemcpyDeviceToDevice, st));
    return AQ_OK;
}

__global__ void k_split_actq(const ActQ* q, int n, float* s, int32_t* z) {
    int i = threadIdx.x;
    if (i < n) {
        if (s) s[i] = q[i].s;
        if (z) z[i] = q[i].z;
    }
}

extern "C" aq_status aq_policy_export_act_qparams(const aq_policy* p, float* d_scale, int32_t* d_zp, void* stream) {
    if (!p) return AQ_EINVAL;
    if (!p->quantized) return AQ_ENOTQUANT;
    hipLaunchKernelGGL(k_split_actq, dim3(1), dim3(64), 0, as_stream(stream), p->actq, p->net.n_layers, d_scale,
                       d_zp);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

// where the one-launch-per-layer plan keeps its intermediate tensors
struct FwdScratch {
    int8_t* i8[2];  // 8-bit activation maps, ping-pong
    float* ln_x;    // fp32 rows into a LayerNorm row kernel
    float* y;       // logits of an argmax head
};

// `fixed`: scratch the caller of this function provides (the allocation-free entry point); NULL = the handle's
// own buffers, grown on demand
static aq_status forward_int8_impl(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                   const aq_taps* taps, const aq_explore* ex, void* stream,
                                   const FwdScratch* fixed = nullptr) {
    if (!p || batch < 0) return AQ_EINVAL;
    if (ex) {
        const aq_status es = explore_args_ok(p, ex, batch);
        if (es != AQ_OK) return es;
    }
    if (!p->quantized) return AQ_ENOTQUANT;
    if (batch == 0) return AQ_OK;
    if (!d_obs || !d_actions) return AQ_EINVAL;
    if (batch > (1LL << 40)) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    const int nl = p->net.n_layers;
    FwdArgs a{};
    a.net = p->h_net;
    a.d_net = p->d_net;
    a.c.obs = d_obs;
    a.c.actions = d_actions;
    a.c.batch = batch;
    a.c.K0 = p->L[0].K;
    a.c.Kp0 = p->L[0].K_pad;
    a.c.in_u8 = p->h_net.in_u8;
    if (p->subbyte && p->w4_slab && p->w4_stale) {
        const aq_status ws = refresh_w4(p, st);
        if (ws != AQ_OK) return ws;
    }
    for (int l = 0; l < nl; ++l) a.w4[l] = p->subbyte ? p->w4[l] : nullptr;
    if (taps) {
        for (int l = 0; l < nl; ++l) {
            a.t.acc[l] = taps->acc ? taps->acc[l] : nullptr;
            a.t.act[l] = taps->act ? taps->act[l] : nullptr;
            a.t.ln[l] = taps->ln_t ? taps->ln_t[l] : nullptr;
        }
        a.t.a0 = taps->a0;
        a.t.y = taps->y;
    }

    int rows;
    size_t lds;
    const bool can_fuse = fused_mlp_supported(a, &rows, &lds);
    if (p->path == 1 && !can_fuse) return AQ_ESHAPE;
    // an MLP that fits the fused kernel always runs fused: measured faster than one launch per layer at
    // every batch size (activations stay in LDS, one launch)
    const int A = p->L.back().N * p->L.back().oh * p->L.back().ow;
    if (can_fuse && p->path != 2) {
        // Gaussian noise rides in the kernel where it writes the actions itself (an elementwise head on
        // a narrow last layer); every other case takes the separate exploration launch below
        const bool fuse_ex = ex && p->net.head != AQ_HEAD_ARGMAX && p->L.back().NT <= 2;
        if (fuse_ex) {
            a.c.ex_sigma = ex->d_sigma;
            a.c.ex_k0 = (uint32_t)ex->seed;
            a.c.ex_k1 = (uint32_t)(ex->seed >> 32);
            a.c.ex_s0 = (uint32_t)ex->step;
            a.c.ex_s1 = (uint32_t)(ex->step >> 32);
        }
        const aq_status fs = launch_fused_mlp(a, st);
        if (fs != AQ_OK || !ex || fuse_ex) return fs;
        return launch_explore(d_actions, batch, A, p->net.head, ex->d_sigma, ex->epsilon, ex->seed, ex->step, st);
    }

    // one launch per layer
    aq_status s = AQ_OK;
    FwdScratch sc;
    if (fixed) {
        sc = *fixed;
    } else {
        s = ensure_i8(p, batch, st);
        if (s != AQ_OK) return s;
        sc = FwdScratch{{p->act_i8[0], p->act_i8[1]}, p->ln_x, p->y_rows};
    }
    if (a.net.in_u8 && a.t.a0) {
        const LayerBuf& b0 = p->L[0];
        const size_t n = (size_t)batch * b0.d.in_h * b0.d.in_w * b0.d.in_c;
        AQ_HIP_CHECK(hipMemcpyAsync(a.t.a0, d_obs, n, hipMemcpyDeviceToDevice, st));
        a.t.a0 = nullptr;
    }
    // the dequantized last-layer rows are only materialised for the y tap or for an argmax head
    float* ybuf = a.t.y ? a.t.y : (p->net.head == AQ_HEAD_ARGMAX ? sc.y : nullptr);
    // a frame policy's convolutions run as one launch where their shapes allow it
    const int nc = p->conv_stack ? conv_stack_layers(a) : 0;
    if (nc) {
        s = launch_conv_stack(a, sc.i8[(nc - 1) & 1], st);
        if (s != AQ_OK) return s;
    }
    for (int l = nc; l < nl; ++l) {
        const LayerBuf& b = p->L[l];
        const int64_t rows_l = batch * b.oh * b.ow;
        LayerIO io;
        io.in = l == 0 ? d_obs : (const void*)sc.i8[(l - 1) & 1];
        io.out = sc.i8[l & 1];
        io.ln_x = sc.ln_x;
        io.y = ybuf;
        s = launch_layer_int8(a, l, io, st);
        if (s != AQ_OK) return s;
        if (l < nl - 1 && b.d.act == AQ_ACT_LN_TANH) {
            s = launch_ln_tanh_rows(a, l, io.ln_x, io.out, rows_l, st);
            if (s != AQ_OK) return s;
        }
        if (l == nl - 1 && p->net.head == AQ_HEAD_ARGMAX && !(layer_uses_skinny(a, l) && skinny_layer_does_argmax(a, l))) {
            s = launch_head_rows(ybuf, rows_l, b.N, p->net.head, d_actions, st);
            if (s != AQ_OK) return s;
        }
    }
    if (ex) return launch_explore(d_actions, batch, A, p->net.head, ex->d_sigma, ex->epsilon, ex->seed, ex->step, st);
    return AQ_OK;
}

extern "C" aq_status aq_policy_forward_int8(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                            const aq_taps* taps, void* stream) {
    return forward_int8_impl(p, d_obs, batch, d_actions, taps, nullptr, stream);
}

extern "C" aq_status aq_policy_step_int8(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                         const aq_explore* ex, const aq_taps* taps, void* stream) {
    return forward_int8_impl(p, d_obs, batch, d_actions, taps, ex, stream);
}

extern "C" aq_status aq_policy_forward_int8_static(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                                   void* stream) {
    if (!p || batch < 0) return AQ_EINVAL;
    unsigned char* base = nullptr;
    const aq_status ss = static_scratch(&base);
    if (ss != AQ_OK) return ss;
    // carve the static array: two 8-bit maps, LayerNorm rows, argmax logits (each piece 256-byte aligned)
    auto up = [](size_t n) { return (n + 255) / 256 * 256; };
    const size_t map = up(i8_map_bytes(p, batch));
    const size_t ln = up((size_t)batch * (size_t)p->ln_elems * 4);
    const size_t y = up((size_t)batch * (size_t)p->y_elems * 4);
    FwdArgs probe{};
    probe.net = p->h_net;
    probe.c.batch = batch > 0 ? batch : 1;
    int rows = 0;
    size_t lds = 0;
    const bool fused = p->path != 2 && fused_mlp_supported(probe, &rows, &lds);
    FwdScratch sc{{nullptr, nullptr}, nullptr, nullptr};
    if (!fused) {  // (the whole-network kernel keeps everything in LDS and needs none of it)
        if ((double)batch * (double)(p->max_hidden_elems + 4 * (p->ln_elems + p->y_elems)) > 1e12 ||
            2 * map + ln + y > (size_t)AQ_STATIC_SCRATCH_BYTES)
            return AQ_ETOOBIG;
        sc.i8[0] = (int8_t*)base;
        sc.i8[1] = (int8_t*)(base + map);
        sc.ln_x = (float*)(base + 2 * map);
        sc.y = (float*)(base + 2 * map + ln);
    }
    return forward_int8_impl(p, d_obs, batch, d_actions, nullptr, nullptr, stream, &sc);
}

// The fp32 actor on explicit parameter arrays.  d_actions may be NULL (calibration only: the head is skipped).
static aq_status forward_fp32_impl(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                   const float* const* h_d_gamma, const float* const* h_d_beta, const void* d_obs,
                                   int64_t batch, void* d_actions, float* d_ranges_out, hipStream_t st) {
    const int nl = p->net.n_layers;
    aq_status s = ensure_f32(p, batch, st);
    if (s != AQ_OK) return s;
    const int in_u8 = p->net.in_type == AQ_IN_U8;
    if (d_ranges_out) {
        s = launch_init_keys(p->keys, nl, st);
        if (s != AQ_OK) return s;
        const LayerBuf& b0 = p->L[0];
        s = launch_minmax_keys(d_obs, in_u8, batch * (int64_t)b0.d.in_h * b0.d.in_w * b0.d.in_c, p->keys, st);
        if (s != AQ_OK) return s;
    }
    for (int l = 0; l < nl; ++l) {
        const LayerBuf& b = p->L[l];
        const bool last = l == nl - 1;
        if (last && !d_actions) break;
        Fp32Layer L{};
        L.w = h_d_w[l];
        L.b = h_d_b ? h_d_b[l] : nullptr;
        L.gamma = h_d_gamma ? h_d_gamma[l] : nullptr;
        L.beta = h_d_beta ? h_d_beta[l] : nullptr;
        L.K = b.K;
        L.N = b.N;
        L.act = b.d.act;
        L.in_h = b.d.in_h;
        L.in_w = b.d.in_w;
        L.in_c = b.d.in_c;
        L.kh = b.d.kh;
        L.kw = b.d.kw;
        L.stride = b.d.stride;
        L.oh = b.oh;
        L.ow = b.ow;
        const int64_t rows_l = batch * b.oh * b.ow;
        const void* in = l == 0 ? d_obs : (const void*)p->act_f32[(l - 1) & 1];
        float* out = p->act_f32[l & 1];
        s = launch_fp32_layer(L, in, l == 0 ? in_u8 : 0, out, rows_l, !last && b.d.act == AQ_ACT_RELU, st);
        if (s != AQ_OK) return s;
        if (!last && b.d.act == AQ_ACT_LN_TANH) {
            s = launch_fp32_ln_tanh(out, rows_l, b.N, L.gamma, L.beta, p->net.ln_eps, st);
            if (s != AQ_OK) return s;
        }
        if (!last && d_ranges_out) {
            s = launch_minmax_keys(out, 0, rows_l * b.N, p->keys + 2 * (l + 1), st);
            if (s != AQ_OK) return s;
        }
        if (last) {
            s = launch_fp32_head(out, rows_l, b.N, p->net.head, d_actions, st);
            if (s != AQ_OK) return s;
        }
    }
    if (d_ranges_out) {
        s = launch_keys_to_ranges(p->keys, 2 * nl, d_ranges_out, st);
        if (s != AQ_OK) return s;
    }
    return AQ_OK;
}

extern "C" aq_status aq_policy_forward_fp32_params(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                                   const float* const* h_d_gamma, const float* const* h_d_beta,
                                                   const void* d_obs, int64_t batch, void* d_actions,
                                                   float* d_ranges_out, void* stream) {
    if (!p || !h_d_w || batch < 0) return AQ_EINVAL;
    if (batch == 0) return AQ_OK;
    if (!d_obs || !d_actions) return AQ_EINVAL;
    for (int l = 0; l < p->net.n_layers; ++l)
        if (!h_d_w[l]) return AQ_EINVAL;
    return forward_fp32_impl(p, h_d_w, h_d_b, h_d_gamma, h_d_beta, d_obs, batch, d_actions, d_ranges_out,
                             as_stream(stream));
}

extern "C" aq_status aq_policy_set_params_fp32(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                               const float* const* h_d_gamma, const float* const* h_d_beta,
                                               void* stream) {
    if (!p || !h_d_w) return AQ_EINVAL;
    const int nl = p->net.n_layers;
    for (int l = 0; l < nl; ++l)
        if (!h_d_w[l]) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    if (!p->f32_slab) {
        if (capturing(st)) return AQ_ETOOBIG;
        size_t bytes = 0;
        std::vector<size_t> offs;
        auto take = [&](size_t n) {
            size_t off = bytes;
            bytes += (n + 255) / 256 * 256;
            return off;
        };
        for (const LayerBuf& b : p->L) {
            offs.push_back(take((size_t)b.N * b.K * 4));
            for (int i = 0; i < 3; ++i) offs.push_back(take((size_t)b.N * 4));
        }
        if (hipMalloc(&p->f32_slab, bytes) != hipSuccess) return AQ_ENOMEM;
        char* base = (char*)p->f32_slab;
        size_t oi = 0;
        for (int l = 0; l < nl; ++l) {
            p->f32_w.push_back((float*)(base + offs[oi++]));
            p->f32_b.push_back((float*)(base + offs[oi++]));
            p->f32_gamma.push_back((float*)(base + offs[oi++]));
            p->f32_beta.push_back((float*)(base + offs[oi++]));
        }
    }
    for (int l = 0; l < nl; ++l) {
        const LayerBuf& b = p->L[l];
        const size_t nb = (size_t)b.N * 4;
        AQ_HIP_CHECK(hipMemcpyAsync(p->f32_w[l], h_d_w[l], (size_t)b.N * b.K * 4, hipMemcpyDeviceToDevice, st));
        // absent biases, gains and offsets take their defaults (0, 1, 0), written by a fill launch
        if (h_d_b && h_d_b[l]) AQ_HIP_CHECK(hipMemcpyAsync(p->f32_b[l], h_d_b[l], nb, hipMemcpyDeviceToDevice, st));
        else if (launch_fill_u32((uint32_t*)p->f32_b[l], b.N, 0u, st) != AQ_OK) return AQ_EHIP;
        if (h_d_gamma && h_d_gamma[l]) AQ_HIP_CHECK(hipMemcpyAsync(p->f32_gamma[l], h_d_gamma[l], nb, hipMemcpyDeviceToDevice, st));
        else if (launch_fill_u32((uint32_t*)p->f32_gamma[l], b.N, 0x3f800000u, st) != AQ_OK) return AQ_EHIP;
        if (h_d_beta && h_d_beta[l]) AQ_HIP_CHECK(hipMemcpyAsync(p->f32_beta[l], h_d_beta[l], nb, hipMemcpyDeviceToDevice, st));
        else if (launch_fill_u32((uint32_t*)p->f32_beta[l], b.N, 0u, st) != AQ_OK) return AQ_EHIP;
    }
    p->f32_ready = true;
    return AQ_OK;
}

extern "C" aq_status aq_policy_forward_fp32(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                            void* stream) {
    if (!p || batch < 0) return AQ_EINVAL;
    if (!p->f32_ready) return AQ_ENOTQUANT;
    if (batch == 0) return AQ_OK;
    if (!d_obs || !d_actions) return AQ_EINVAL;
    return forward_fp32_impl(p, p->f32_w.data(), p->f32_b.data(), p->f32_gamma.data(), p->f32_beta.data(), d_obs, batch,
                             d_actions, nullptr, as_stream(stream));
}

extern "C" aq_status aq_calibrate_fp32(aq_policy* p, const void* d_obs, int64_t batch, aq_range* h_ranges_out,
                                       void* stream) {
    if (!p || !d_obs || !h_ranges_out || batch < 1) return AQ_EINVAL;
    if (!p->f32_ready) return AQ_ENOTQUANT;
    hipStream_t st = as_stream(stream);
    if (capturing(st)) return AQ_EINVAL;  // the call has to wait for its result
    const aq_status s = forward_fp32_impl(p, p->f32_w.data(), p->f32_b.data(), p->f32_gamma.data(), p->f32_beta.data(),
                                          d_obs, batch, nullptr, p->calib, st);
    if (s != AQ_OK) return s;
    float h[2 * AQ_MAX_LAYERS];
    const int nl = p->net.n_layers;
    AQ_HIP_CHECK(hipMemcpyAsync(h, p->calib, sizeof(float) * 2 * nl, hipMemcpyDeviceToHost, st));
    AQ_HIP_CHECK(hipStreamSynchronize(st));
    for (int l = 0; l < nl; ++l) {
        h_ranges_out[l].lo = h[2 * l];
        h_ranges_out[l].hi = h[2 * l + 1];
    }
    return AQ_OK;
}

// ---- half-precision actor
extern "C" aq_status aq_convert_params_fp16(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                            const float* const* h_d_gamma, const float* const* h_d_beta,
                                            void* stream) {
    if (!p || !h_d_w) return AQ_EINVAL;
    const int nl = p->net.n_layers;
    for (int l = 0; l < nl; ++l)
        if (!h_d_w[l]) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    if (!p->h16_slab) {
        size_t bytes = 0;
        std::vector<size_t> offs;
        auto take = [&](size_t n) {
            size_t off = bytes;
            bytes += (n + 255) / 256 * 256;
            return off;
        };
        for (const LayerBuf& b : p->L) {
            const int ks16 = round_up(b.K, 64) / 16;
            offs.push_back(take((size_t)b.NT * ks16 * 1024));
            for (int i = 0; i < 3; ++i) offs.push_back(take((size_t)b.N_pad * 4));
        }
        if (hipMalloc(&p->h16_slab, bytes) != hipSuccess) return AQ_ENOMEM;
        char* base = (char*)p->h16_slab;
        size_t oi = 0;
        for (int l = 0; l < nl; ++l) {
            p->h16_wp.push_back(base + offs[oi++]);
            p->h16_bias.push_back((float*)(base + offs[oi++]));
            p->h16_gamma.push_back((float*)(base + offs[oi++]));
            p->h16_beta.push_back((float*)(base + offs[oi++]));
        }
    }
    int* st16 = p->status + 1;
    aq_status s = launch_fill_u32((uint32_t*)st16, 1, 0u, st);
    if (s != AQ_OK) return s;
    for (int l = 0; l < nl; ++l) {
        const LayerBuf& b = p->L[l];
        const int ks16 = round_up(b.K, 64) / 16;
        s = launch_fp16_pack_weights(h_d_w[l], b.N, b.K, ks16, b.NT, p->h16_wp[l], st16, st);
        if (s != AQ_OK) return s;
        s = launch_fp16_round_vec(h_d_b ? h_d_b[l] : nullptr, b.N, b.N_pad, 0.0f, p->h16_bias[l], st16, st);
        if (s != AQ_OK) return s;
        if (b.d.act == AQ_ACT_LN_TANH) {
            s = launch_fp16_round_vec(h_d_gamma ? h_d_gamma[l] : nullptr, b.N, b.N_pad, 1.0f, p->h16_gamma[l], st16, st);
            if (s != AQ_OK) return s;
            s = launch_fp16_round_vec(h_d_beta ? h_d_beta[l] : nullptr, b.N, b.N_pad, 0.0f, p->h16_beta[l], st16, st);
            if (s != AQ_OK) return s;
        }
    }
    p->h16_ready = true;
    return AQ_OK;
}

static void fp16_layers(const aq_policy* p, Fp16Layer* Ls) {
    const int nl = p->net.n_layers;
    for (int l = 0; l < nl; ++l) {
        const LayerBuf& b = p->L[l];
        const bool last = l == nl - 1;
        Fp16Layer L{};
        L.wp = p->h16_ready ? p->h16_wp[l] : nullptr;
        L.bias = p->h16_ready ? p->h16_bias[l] : nullptr;
        L.K = b.K;
        L.N = b.N;
        L.KS16 = round_up(b.K, 64) / 16;
        L.NT = b.NT;
        L.fc = b.fc;
        L.relu = !last && b.d.act == AQ_ACT_RELU;
        L.in_h = b.d.in_h;
        L.in_w = b.d.in_w;
        L.in_c = b.d.in_c;
        L.kh = b.d.kh;
        L.kw = b.d.kw;
        L.stride = b.d.stride;
        L.oh = b.oh;
        L.ow = b.ow;
        Ls[l] = L;
    }
}

extern "C" aq_status aq_policy_fp16_conv_stack_layers(const aq_policy* p, int32_t* n_layers) {
    if (!p || !n_layers) return AQ_EINVAL;
    Fp16Layer Ls[AQ_MAX_LAYERS];
    fp16_layers(p, Ls);
    *n_layers = p->conv_stack ? fp16_conv_stack_layers(Ls, p->net.n_layers, nullptr,
                                                       p->net.in_type == AQ_IN_U8 ? 2 : 1, 1)
                              : 0;
    return AQ_OK;
}

extern "C" aq_status aq_policy_forward_fp16(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                            void* const* taps_out, void* stream) {
    if (!p || batch < 0) return AQ_EINVAL;
    if (!p->h16_ready) return AQ_ENOTQUANT;
    if (batch == 0) return AQ_OK;
    if (!d_obs || !d_actions) return AQ_EINVAL;
    hipStream_t st = as_stream(stream);
    aq_status s = ensure_f16(p, batch, st);
    if (s != AQ_OK) return s;
    const int nl = p->net.n_layers;
    const int in_mode0 = p->net.in_type == AQ_IN_U8 ? 2 : 1;
    Fp16Layer Ls[AQ_MAX_LAYERS];
    fp16_layers(p, Ls);
    // a frame policy's convolutions run as one launch where their shapes allow it (their maps then stay in
    // LDS, so a tap on any but the last of them takes the per-layer launches)
    int nc = p->conv_stack ? fp16_conv_stack_layers(Ls, nl, d_obs, in_mode0, batch) : 0;
    for (int l = 0; l + 1 < nc; ++l)
        if (taps_out && taps_out[l]) nc = 0;
    if (nc) {
        const LayerBuf& b = p->L[nc - 1];
        void* out = p->act_f16[(nc - 1) & 1];
        s = launch_fp16_conv_stack(Ls, nl, d_obs, in_mode0, batch, out, st);
        if (s != AQ_OK) return s;
        if (taps_out && taps_out[nc - 1])
            AQ_HIP_CHECK(hipMemcpyAsync(taps_out[nc - 1], out, (size_t)batch * b.oh * b.ow * b.N * 2,
                                        hipMemcpyDeviceToDevice, st));
    }
    for (int l = nc; l < nl; ++l) {
        const LayerBuf& b = p->L[l];
        const bool last = l == nl - 1;
        Fp16Layer L = Ls[l];
        const int64_t rows_l = batch * b.oh * b.ow;
        const void* in = l == 0 ? d_obs : (const void*)p->act_f16[(l - 1) & 1];
        void* out = p->act_f16[l & 1];
        // (the layer kernel writes actions in 16-byte pieces)
        const bool fused_head = last && p->net.head != AQ_HEAD_ARGMAX && ((uintptr_t)d_actions & 15) == 0;
        if (fused_head) {
            L.head_actions = (float*)d_actions;
            L.head_tanh = p->net.head == AQ_HEAD_TANH;
        }
        // an argmax policy whose logits fit one tile of the few-row kernel: the action index leaves the same launch
        const bool fused_argmax = last && p->net.head == AQ_HEAD_ARGMAX && L.NT == 1 &&
                                  fp16_layer_is_skinny(L, in, l == 0 ? in_mode0 : 0, rows_l);
        if (fused_argmax) L.head_argmax = (int32_t*)d_actions;
        s = launch_layer_fp16(L, in, l == 0 ? in_mode0 : 0, out, rows_l, st);
        if (s != AQ_OK) return s;
        if (!last && b.d.act == AQ_ACT_LN_TANH) {
            s = launch_fp16_ln_tanh(out, rows_l, b.N, p->h16_gamma[l], p->h16_beta[l], p->net.ln_eps, st);
            if (s != AQ_OK) return s;
        }
        if (taps_out && taps_out[l])
            AQ_HIP_CHECK(hipMemcpyAsync(taps_out[l], out, (size_t)rows_l * b.N * 2, hipMemcpyDeviceToDevice, st));
        if (last && !fused_head && !fused_argmax) {
            s = launch_fp16_head(out, rows_l, b.N, p->net.head, d_actions, st);
            if (s != AQ_OK) return s;
        }
    }
    return AQ_OK;
}
