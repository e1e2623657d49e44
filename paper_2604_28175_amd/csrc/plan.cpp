// Model load (paper Section 3, first paragraph after Figure 3: models are loaded and their
// instances initialised before serving) and the per-batch kernel sequence (Section 3.2 step (2)).
//
// Load: parse the weight container, fold BatchNorm into the preceding convolution in fp32
// (scale = gamma / sqrt(var + 1e-5); w' = fp16(w * scale); b' = beta - mean * scale), re-lay
// OIHW weights as [K][R][S][C] to match NHWC activations, upload, and lay out the layer plan.
// Run: enqueue every layer of the plan on one stream, no host synchronisation in between.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "runtime.hpp"

namespace strait {

static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
const char* last_error() { return g_err; }

#define HIP_TRY(expr)                                                                   \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) { set_error("%s: %s", #expr, hipGetErrorString(e_)); return STRAIT_E_HIP; } \
    } while (0)

// ------------------------------------------------------------------------------------------
// container
struct TensorView { const half_t* data; int ndim; unsigned shape[4]; size_t count; };

struct Container {
    int arch = 0;
    unsigned hyper[8] = {0};
    std::map<std::string, TensorView> t;
    const TensorView* find(const std::string& name) const {
        auto it = t.find(name);
        if (it == t.end()) { set_error("weight container: tensor '%s' missing", name.c_str()); return nullptr; }
        return &it->second;
    }
};

static int parse_container(const void* blob, size_t bytes, Container& c) {
    const unsigned char* p = (const unsigned char*)blob;
    if (!p || bytes < 48 || memcmp(p, "STRW", 4) != 0) { set_error("weight container: bad magic"); return STRAIT_E_FORMAT; }
    unsigned head[11];
    memcpy(head, p + 4, sizeof(head));
    if (head[0] != 1) { set_error("weight container: unsupported version %u", head[0]); return STRAIT_E_FORMAT; }
    c.arch = (int)head[1];
    const unsigned n = head[2];
    memcpy(c.hyper, head + 3, 32);
    if ((size_t)48 + (size_t)n * 80 > bytes) { set_error("weight container: truncated table"); return STRAIT_E_FORMAT; }
    for (unsigned i = 0; i < n; ++i) {
        const unsigned char* e = p + 48 + (size_t)i * 80;
        char name[41];
        memcpy(name, e, 40);
        name[40] = 0;
        unsigned meta[6];
        memcpy(meta, e + 40, 24);
        unsigned long long off, nb;
        memcpy(&off, e + 64, 8);
        memcpy(&nb, e + 72, 8);
        TensorView v;
        v.ndim = (int)meta[1];
        if (meta[0] != 0 || v.ndim < 1 || v.ndim > 4) { set_error("weight container: tensor '%s' has unsupported dtype/rank", name); return STRAIT_E_FORMAT; }
        v.count = 1;
        for (int d = 0; d < 4; ++d) { v.shape[d] = meta[2 + d]; if (d < v.ndim) v.count *= v.shape[d]; }
        if (nb != v.count * 2 || off % 2 != 0 || off > bytes || nb > bytes - off) { set_error("weight container: tensor '%s' out of bounds", name); return STRAIT_E_FORMAT; }
        v.data = (const half_t*)(p + off);
        c.t[name] = v;
    }
    return 0;
}

// ------------------------------------------------------------------------------------------
// weight preparation (host) + upload
struct Loader {
    Model& m;
    const Container& c;
    int upload(const void* host, size_t bytes, void** dev) {
        void* d = nullptr;
        const size_t padded = (bytes + 255) / 256 * 256;
        if (hipMalloc(&d, padded) != hipSuccess) { set_error("hipMalloc(%zu) for weights failed", padded); return STRAIT_E_NOMEM; }
        m.dev_allocs.push_back(d);
        HIP_TRY(hipMemset(d, 0, padded));
        HIP_TRY(hipMemcpy(d, host, bytes, hipMemcpyHostToDevice));
        *dev = d;
        return 0;
    }
    static bool shape_is(const TensorView* v, std::initializer_list<unsigned> s) {
        if (!v || v->ndim != (int)s.size()) return false;
        int i = 0;
        for (unsigned d : s) if (v->shape[i++] != d) return false;
        return true;
    }
    // per-output-channel scale and bias: BatchNorm fold, or plain bias tensor, in fp32
    int scale_bias(const std::string& name, bool bn, unsigned K, std::vector<float>& scale, std::vector<float>& bias) {
        scale.assign(K, 1.f);
        bias.assign(K, 0.f);
        if (bn) {
            const TensorView *g = c.find(name + ".gamma"), *b = c.find(name + ".beta"), *mu = c.find(name + ".mean"), *var = c.find(name + ".var");
            if (!g || !b || !mu || !var) return STRAIT_E_FORMAT;
            if (!shape_is(g, {K}) || !shape_is(b, {K}) || !shape_is(mu, {K}) || !shape_is(var, {K})) { set_error("'%s': BatchNorm vectors must have %u entries", name.c_str(), K); return STRAIT_E_FORMAT; }
            for (unsigned k = 0; k < K; ++k) {
                const float s = (float)g->data[k] / sqrtf((float)var->data[k] + 1e-5f);
                volatile float ms = (float)mu->data[k] * s;       // two roundings: no fused multiply-add
                scale[k] = s;
                bias[k] = (float)b->data[k] - ms;
            }
        } else {
            const TensorView* b = c.find(name + ".b");
            if (!b) return STRAIT_E_FORMAT;
            if (!shape_is(b, {K})) { set_error("'%s.b': expected %u entries", name.c_str(), K); return STRAIT_E_FORMAT; }
            for (unsigned k = 0; k < K; ++k) bias[k] = (float)b->data[k];
        }
        return 0;
    }
    // OIHW [K][C][R][S] -> [K][R][S][C] with the fold scale applied, row pitch ldw (>= R*S*C, zero padded)
    int conv_weights(const std::string& name, bool bn, unsigned K, unsigned C, unsigned R, unsigned S, Op& op) {
        const TensorView* w = c.find(name + ".w");
        if (!w) return STRAIT_E_FORMAT;
        if (!shape_is(w, {K, C, R, S})) { set_error("'%s.w': expected [%u,%u,%u,%u]", name.c_str(), K, C, R, S); return STRAIT_E_FORMAT; }
        std::vector<float> scale, bias;
        int rc = scale_bias(name, bn, K, scale, bias);
        if (rc) return rc;
        const unsigned Kg = R * S * C, ldw = (Kg + 7) / 8 * 8;
        std::vector<half_t> out((size_t)K * ldw, (half_t)0);
        for (unsigned k = 0; k < K; ++k)
            for (unsigned cc = 0; cc < C; ++cc)
                for (unsigned r = 0; r < R; ++r)
                    for (unsigned s = 0; s < S; ++s) {
                        const float v = (float)w->data[((k * C + cc) * R + r) * S + s];
                        out[(size_t)k * ldw + (r * S + s) * C + cc] = bn ? (half_t)(v * scale[k]) : (half_t)v;
                    }
        void *dw = nullptr, *db = nullptr;
        if ((rc = upload(out.data(), out.size() * 2, &dw))) return rc;
        if ((rc = upload(bias.data(), bias.size() * 4, &db))) return rc;
        op.w = (const half_t*)dw;
        op.bias = (const float*)db;
        op.ldw = (int)ldw;
        op.info.weight_bytes = (int64_t)K * Kg * 2 + K * 4;
        return 0;
    }
    // A block-closing 1x1 convolution and the 1x1 projection shortcut beside it as one weight matrix [K][C1 + C2] (each
    // half folded and rounded exactly as conv_weights does it) and one bias (the two folded biases added in fp32).
    int proj_pair_weights(const std::string& n3, unsigned C1, const std::string& nd, unsigned C2, unsigned K, Op& op) {
        const unsigned ldw = C1 + C2;
        std::vector<half_t> out((size_t)K * ldw, (half_t)0);
        std::vector<float> bsum(K, 0.f);
        unsigned off = 0;
        for (int part = 0; part < 2; ++part) {
            const std::string& name = part ? nd : n3;
            const unsigned C = part ? C2 : C1;
            const TensorView* w = c.find(name + ".w");
            if (!w) return STRAIT_E_FORMAT;
            if (!shape_is(w, {K, C, 1, 1})) { set_error("'%s.w': expected [%u,%u,1,1]", name.c_str(), K, C); return STRAIT_E_FORMAT; }
            std::vector<float> scale, bias;
            int rc = scale_bias(name, true, K, scale, bias);
            if (rc) return rc;
            for (unsigned k = 0; k < K; ++k) {
                for (unsigned cc = 0; cc < C; ++cc) out[(size_t)k * ldw + off + cc] = (half_t)((float)w->data[k * C + cc] * scale[k]);
                bsum[k] += bias[k];
            }
            off += C;
        }
        void *dw = nullptr, *db = nullptr;
        int rc;
        if ((rc = upload(out.data(), out.size() * 2, &dw))) return rc;
        if ((rc = upload(bsum.data(), bsum.size() * 4, &db))) return rc;
        op.w_proj = (const half_t*)dw;
        op.bias_proj = (const float*)db;
        return 0;
    }
    // Stem: OIHW [K][C][R][S] -> [K][R][Sv*Cpad] with taps s >= S and channels c >= C zero.
    int stem_weights(const std::string& name, bool bn, unsigned K, unsigned C, unsigned R, unsigned S, unsigned Sv, unsigned Cpad, Op& op) {
        const TensorView* w = c.find(name + ".w");
        if (!w) return STRAIT_E_FORMAT;
        if (!shape_is(w, {K, C, R, S})) { set_error("'%s.w': expected [%u,%u,%u,%u]", name.c_str(), K, C, R, S); return STRAIT_E_FORMAT; }
        std::vector<float> scale, bias;
        int rc = scale_bias(name, bn, K, scale, bias);
        if (rc) return rc;
        const unsigned Cv = Sv * Cpad, ldw = R * Cv;
        std::vector<half_t> out((size_t)K * ldw, (half_t)0);
        for (unsigned k = 0; k < K; ++k)
            for (unsigned cc = 0; cc < C; ++cc)
                for (unsigned r = 0; r < R; ++r)
                    for (unsigned s = 0; s < S; ++s) {
                        const float v = (float)w->data[((k * C + cc) * R + r) * S + s];
                        out[(size_t)k * ldw + r * Cv + s * Cpad + cc] = bn ? (half_t)(v * scale[k]) : (half_t)v;
                    }
        void *dw = nullptr, *db = nullptr;
        if ((rc = upload(out.data(), out.size() * 2, &dw))) return rc;
        if ((rc = upload(bias.data(), bias.size() * 4, &db))) return rc;
        op.w = (const half_t*)dw;
        op.bias = (const float*)db;
        op.ldw = (int)ldw;
        op.info.weight_bytes = (int64_t)K * C * R * S * 2 + K * 4;
        return 0;
    }
    // Fused stem + pooling: OIHW [64][3][7][7] -> [64][22 fragments][8]; fragment 3r + j = halfs 8j..8j+7 of filter
    // row r's window {0, (s=0: c=0,1,2), ..., (s=6: c=0,1,2), 0, 0}; the 22nd fragment stays zero.
    int stempool_weights(const std::string& name, bool bn, Op& op) {
        const unsigned K = 64, C = 3, R = 7, S = 7;
        const TensorView* w = c.find(name + ".w");
        if (!w) return STRAIT_E_FORMAT;
        if (!shape_is(w, {K, C, R, S})) { set_error("'%s.w': expected [%u,%u,%u,%u]", name.c_str(), K, C, R, S); return STRAIT_E_FORMAT; }
        std::vector<float> scale, bias;
        int rc = scale_bias(name, bn, K, scale, bias);
        if (rc) return rc;
        const unsigned ldw = 22 * 8;
        std::vector<half_t> out((size_t)K * ldw, (half_t)0);
        for (unsigned k = 0; k < K; ++k)
            for (unsigned r = 0; r < R; ++r)
                for (unsigned s = 0; s < S; ++s)
                    for (unsigned cc = 0; cc < C; ++cc) {
                        const float v = (float)w->data[((k * C + cc) * R + r) * S + s];
                        out[(size_t)k * ldw + r * 24 + 1 + s * 3 + cc] = bn ? (half_t)(v * scale[k]) : (half_t)v;
                    }
        void *dw = nullptr, *db = nullptr;
        if ((rc = upload(out.data(), out.size() * 2, &dw))) return rc;
        if ((rc = upload(bias.data(), bias.size() * 4, &db))) return rc;
        op.w = (const half_t*)dw;
        op.bias = (const float*)db;
        op.ldw = (int)ldw;
        op.info.weight_bytes = (int64_t)K * C * R * S * 2 + K * 4;
        return 0;
    }
    // Direct 3x3/2 stem: OIHW [K][3][3][3] -> [32][3 filter rows][16]: a filter row's window {0, (s=0: c=0,1,2), (s=1: ..),
    // (s=2: ..), 0 x 6}; rows from K on stay zero.
    int stem3_weights(const std::string& name, bool bn, unsigned K, Op& op) {
        const unsigned C = 3, R = 3, S = 3;
        const TensorView* w = c.find(name + ".w");
        if (!w) return STRAIT_E_FORMAT;
        if (!shape_is(w, {K, C, R, S})) { set_error("'%s.w': expected [%u,%u,%u,%u]", name.c_str(), K, C, R, S); return STRAIT_E_FORMAT; }
        std::vector<float> scale, bias;
        int rc = scale_bias(name, bn, K, scale, bias);
        if (rc) return rc;
        const unsigned ldw = 48;
        std::vector<half_t> out((size_t)32 * ldw, (half_t)0);
        for (unsigned k = 0; k < K; ++k)
            for (unsigned r = 0; r < R; ++r)
                for (unsigned s = 0; s < S; ++s)
                    for (unsigned cc = 0; cc < C; ++cc) {
                        const float v = (float)w->data[((k * C + cc) * R + r) * S + s];
                        out[(size_t)k * ldw + r * 16 + 1 + s * 3 + cc] = bn ? (half_t)(v * scale[k]) : (half_t)v;
                    }
        void *dw = nullptr, *db = nullptr;
        if ((rc = upload(out.data(), out.size() * 2, &dw))) return rc;
        if ((rc = upload(bias.data(), bias.size() * 4, &db))) return rc;
        op.w = (const half_t*)dw;
        op.bias = (const float*)db;
        op.ldw = (int)ldw;
        op.info.weight_bytes = (int64_t)K * C * R * S * 2 + K * 4;
        return 0;
    }
    // depthwise [C][1][3][3] -> [3][3][C]
    int dw_weights(const std::string& name, unsigned C, Op& op) {
        const TensorView* w = c.find(name + ".w");
        if (!w) return STRAIT_E_FORMAT;
        if (!shape_is(w, {C, 1, 3, 3})) { set_error("'%s.w': expected [%u,1,3,3]", name.c_str(), C); return STRAIT_E_FORMAT; }
        std::vector<float> scale, bias;
        int rc = scale_bias(name, true, C, scale, bias);
        if (rc) return rc;
        std::vector<half_t> out((size_t)9 * C);
        for (unsigned cc = 0; cc < C; ++cc)
            for (unsigned k = 0; k < 9; ++k) out[(size_t)k * C + cc] = (half_t)((float)w->data[cc * 9 + k] * scale[cc]);
        void *dw = nullptr, *db = nullptr;
        if ((rc = upload(out.data(), out.size() * 2, &dw))) return rc;
        if ((rc = upload(bias.data(), bias.size() * 4, &db))) return rc;
        op.w = (const half_t*)dw;
        op.bias = (const float*)db;
        op.info.weight_bytes = (int64_t)C * 9 * 2 + C * 4;
        return 0;
    }
    // linear layers: rows of several [out_i, in] matrices stacked, biases concatenated
    int linear_weights(std::initializer_list<std::string> names, unsigned in, Op& op, unsigned* total_out) {
        std::vector<half_t> w;
        std::vector<float> b;
        for (const std::string& nm : names) {
            const TensorView *tw = c.find(nm + ".w"), *tb = c.find(nm + ".b");
            if (!tw || !tb) return STRAIT_E_FORMAT;
            if (tw->ndim != 2 || tw->shape[1] != in || !shape_is(tb, {tw->shape[0]})) { set_error("'%s': expected [out,%u] weight and [out] bias", nm.c_str(), in); return STRAIT_E_FORMAT; }
            w.insert(w.end(), tw->data, tw->data + tw->count);
            for (unsigned i = 0; i < tb->count; ++i) b.push_back((float)tb->data[i]);
        }
        if (in % 8 != 0) { set_error("linear layer input width %u must be a multiple of 8", in); return STRAIT_E_SHAPE; }
        void *dw = nullptr, *db = nullptr;
        int rc;
        if ((rc = upload(w.data(), w.size() * 2, &dw))) return rc;
        if ((rc = upload(b.data(), b.size() * 4, &db))) return rc;
        op.w = (const half_t*)dw;
        op.bias = (const float*)db;
        op.ldw = (int)in;
        *total_out = (unsigned)b.size();
        op.info.weight_bytes = (int64_t)w.size() * 2 + (int64_t)b.size() * 4;
        return 0;
    }
    int vector_f32(const std::string& name, unsigned n, const float** dev) {
        const TensorView* v = c.find(name);
        if (!v) return STRAIT_E_FORMAT;
        if (!shape_is(v, {n})) { set_error("'%s': expected %u entries", name.c_str(), n); return STRAIT_E_FORMAT; }
        std::vector<float> f(n);
        for (unsigned i = 0; i < n; ++i) f[i] = (float)v->data[i];
        void* d = nullptr;
        int rc = upload(f.data(), f.size() * 4, &d);
        *dev = (const float*)d;
        return rc;
    }
};

// ------------------------------------------------------------------------------------------
// activation buffer planning: a handful of reusable buffers, sized per sample
struct Planner {
    Model& m;
    std::vector<bool> busy;
    int get(size_t elems) {
        int best = -1;
        for (size_t i = 0; i < busy.size(); ++i)
            if (!busy[i] && (best < 0 || m.buf_elems[i] > m.buf_elems[best])) best = (int)i;
        if (best < 0) { m.buf_elems.push_back(0); busy.push_back(false); best = (int)busy.size() - 1; }
        busy[best] = true;
        if (m.buf_elems[best] < elems) m.buf_elems[best] = elems;
        return best;
    }
    void put(int slot) { if (slot >= 0) busy[slot] = false; }
};

static void name_op(Op& op, const std::string& name, int info_kind) {
    op.name = name;
    memset(&op.info, 0, sizeof(op.info));
    snprintf(op.info.name, sizeof(op.info.name), "%s", name.c_str());
    op.info.kind = info_kind;
}

struct Builder {
    Model& m;
    Loader& ld;
    Planner pl;

    static int osz(int h, int k, int stride, int pad) { return (h + 2 * pad - k) / stride + 1; }

    // regular convolution / linear layer on an NHWC activation
    int conv(const std::string& name, bool bn, int in, int H, int W, int C, int K, int R, int stride, int pad, int act,
             int res, int out, int* P_out, int* Q_out) {
        Op op;
        name_op(op, name, 0);
        op.kind = OP_CONV;
        op.in = in; op.out = out; op.res = res;
        op.H = H; op.W = W; op.C = C; op.K = K; op.R = R; op.S = R; op.stride = stride; op.pad = pad; op.act = act;
        op.P = osz(H, R, stride, pad); op.Q = osz(W, R, stride, pad);
        op.vC = C; op.vR = R; op.vS = R; op.vH = H; op.vW = W;
        op.sN = (long long)H * W * C; op.sH = W * C; op.sW = C; op.stride_w = stride; op.pad_h = pad; op.pad_w = pad;
        int rc = ld.conv_weights(name, bn, K, C, R, R, op);
        if (rc) return rc;
        op.info.macs_per_sample = (int64_t)op.P * op.Q * K * R * R * C;
        op.info.bytes_per_sample = 2LL * ((int64_t)H * W * C + (int64_t)op.P * op.Q * K * (res != SLOT_NONE ? 2 : 1));
        op.info.gemm_m_per_sample = op.P * op.Q; op.info.gemm_n = K; op.info.gemm_k = R * R * C;
        if (P_out) *P_out = op.P;
        if (Q_out) *Q_out = op.Q;
        m.ops.push_back(op);
        return 0;
    }

    // 3-channel stem: pack to a zero-bordered, channel-padded image, then a convolution whose
    // row taps are contiguous in memory
    int stem(const std::string& name, bool bn, int H, int W, int C, int K, int R, int stride, int pad, int act, int out_slot_elems_hint,
             int* out_slot, int* P_out, int* Q_out) {
        (void)out_slot_elems_hint;
        if (C == 3 && R == 3 && stride == 2 && pad == 1 && K >= 8 && K <= 32 && K % 8 == 0 && W % 2 == 0 && act != ACT_GELU) {
            // MobileNetV2's stem: a kernel of its own that reads the image as it lies in memory (no packed copy)
            const int P = osz(H, 3, 2, 1), Q = osz(W, 3, 2, 1);
            Op op;
            name_op(op, name, 0);
            op.kind = OP_STEM3;
            op.in = SLOT_INPUT;
            op.H = H; op.W = W; op.C = 3; op.K = K; op.R = op.S = 3; op.stride = 2; op.pad = 1; op.act = act;
            op.P = P; op.Q = Q;
            int rc = ld.stem3_weights(name, bn, (unsigned)K, op);
            if (rc) return rc;
            op.out = pl.get((size_t)P * Q * K);
            op.info.macs_per_sample = (int64_t)P * Q * K * 27;
            op.info.bytes_per_sample = 2LL * ((int64_t)H * W * 3 + (int64_t)P * Q * K);
            op.info.gemm_m_per_sample = P * Q; op.info.gemm_n = K; op.info.gemm_k = 48;
            m.ops.push_back(op);
            *out_slot = op.out; *P_out = P; *Q_out = Q;
            return 0;
        }
        const int Cpad = (stride * 4) % 8 == 0 ? 4 : 8;
        int Sv = R;
        while ((Sv * Cpad) % 32 != 0) ++Sv;       // 32 channels per virtual tap row: the reduction then runs through the LDS-direct kernel
        const int P = osz(H, R, stride, pad), Q = osz(W, R, stride, pad);
        int Hp = std::max(H + 2 * pad, (P - 1) * stride + R);
        int Wp = std::max(W + 2 * pad, (Q - 1) * stride + Sv);
        while ((Wp * Cpad) % 8 != 0) ++Wp;
        const int pk = pl.get((size_t)Hp * Wp * Cpad);
        Op pack;
        name_op(pack, name + ".pack", 6);
        pack.kind = OP_PACK;
        pack.in = SLOT_INPUT; pack.out = pk;
        pack.H = H; pack.W = W; pack.C = C; pack.Hp = Hp; pack.Wp = Wp; pack.Cpad = Cpad; pack.pad = pad;
        pack.P = Hp; pack.Q = Wp; pack.K = Cpad;
        pack.info.bytes_per_sample = 2LL * ((int64_t)H * W * C + (int64_t)Hp * Wp * Cpad);
        m.ops.push_back(pack);

        Op op;
        name_op(op, name, 0);
        op.kind = OP_CONV;
        op.in = pk; op.res = SLOT_NONE;
        op.H = H; op.W = W; op.C = C; op.K = K; op.R = R; op.S = R; op.stride = stride; op.pad = pad; op.act = act;
        op.P = P; op.Q = Q;
        op.vC = Sv * Cpad; op.vR = R; op.vS = 1; op.vH = Hp; op.vW = Q;
        op.sN = (long long)Hp * Wp * Cpad; op.sH = Wp * Cpad; op.sW = stride * Cpad; op.stride_w = 1; op.pad_h = 0; op.pad_w = 0;
        int rc = ld.stem_weights(name, bn, K, C, R, R, Sv, Cpad, op);
        if (rc) return rc;
        op.out = pl.get((size_t)P * Q * K);
        pl.put(pk);
        op.info.macs_per_sample = (int64_t)P * Q * K * R * R * C;
        op.info.bytes_per_sample = 2LL * ((int64_t)Hp * Wp * Cpad + (int64_t)P * Q * K);
        op.info.gemm_m_per_sample = P * Q; op.info.gemm_n = K; op.info.gemm_k = R * op.vC;
        m.ops.push_back(op);
        *out_slot = op.out; *P_out = P; *Q_out = Q;
        return 0;
    }

    // ResNet's 7x7/2 stem convolution (+ ReLU) and the 3x3/2 max pooling behind it as one launch
    int stem_pool(const std::string& name, bool bn, int H, int W, int* out_slot, int* P_out, int* Q_out) {
        const int P = osz(H, 7, 2, 3), Q = osz(W, 7, 2, 3), P2 = osz(P, 3, 2, 1), Q2 = osz(Q, 3, 2, 1);
        Op op;
        name_op(op, name, 0);
        op.kind = OP_STEMPOOL;
        op.in = SLOT_INPUT;
        op.H = H; op.W = W; op.C = 3; op.K = 64; op.R = op.S = 7; op.stride = 2; op.pad = 3; op.act = ACT_RELU;
        op.P = P2; op.Q = Q2;
        int rc = ld.stempool_weights("stem", bn, op);
        if (rc) return rc;
        op.out = pl.get((size_t)P2 * Q2 * 64);
        op.info.macs_per_sample = (int64_t)P * Q * 64 * 7 * 7 * 3;
        op.info.bytes_per_sample = 2LL * ((int64_t)H * W * 3 + (int64_t)P2 * Q2 * 64);
        op.info.gemm_m_per_sample = P * Q; op.info.gemm_n = 64; op.info.gemm_k = 7 * 24;
        m.ops.push_back(op);
        *out_slot = op.out; *P_out = P2; *Q_out = Q2;
        return 0;
    }

    int dwconv(const std::string& name, int in, int H, int W, int C, int stride, int out, int* P_out, int* Q_out) {
        Op op;
        name_op(op, name, 1);
        op.kind = OP_DWCONV;
        op.in = in; op.out = out;
        op.H = H; op.W = W; op.C = C; op.K = C; op.R = op.S = 3; op.stride = stride; op.pad = 1; op.act = ACT_RELU6;
        op.P = osz(H, 3, stride, 1); op.Q = osz(W, 3, stride, 1);
        int rc = ld.dw_weights(name, C, op);
        if (rc) return rc;
        op.info.macs_per_sample = (int64_t)op.P * op.Q * C * 9;
        op.info.bytes_per_sample = 2LL * ((int64_t)H * W * C + (int64_t)op.P * op.Q * C);
        *P_out = op.P; *Q_out = op.Q;
        m.ops.push_back(op);
        return 0;
    }

    void pool(const std::string& name, int sub, int in, int H, int W, int C, int out, int out_ref = 0) {
        Op op;
        name_op(op, name, 2);
        op.kind = OP_POOL; op.sub = sub;
        op.in = in; op.out = out; op.out_ref = out_ref;
        op.H = H; op.W = W; op.C = C; op.K = C;
        if (sub == POOL_MAX3X3S2) { op.P = osz(H, 3, 2, 1); op.Q = osz(W, 3, 2, 1); }
        if (sub == POOL_MAX2X2S2) { op.P = H / 2; op.Q = W / 2; }
        op.info.bytes_per_sample = 2LL * ((int64_t)H * W * C + (int64_t)op.P * op.Q * C);
        m.ops.push_back(op);
    }

    // GAP -> FC (fp32 logits into the output buffer) -> softmax + top-1
    int classifier(int feat_in, int HW_h, int HW_w, int C, int classes) {
        const int f = pl.get(C);
        pool("gap", POOL_GLOBAL_AVG, feat_in, HW_h, HW_w, C, f);
        pl.put(feat_in);
        return head(f, C, classes);
    }

    // a plain linear layer on one feature vector per sample: y = act(x W^T + b), fp16
    int dense(const std::string& name, int in, int C, int K, int act, int out) {
        Op op;
        name_op(op, name, 0);
        op.kind = OP_CONV;
        op.in = in; op.out = out; op.act = act;
        op.C = C; op.K = K; op.vC = C; op.vR = op.vS = 1; op.vH = op.vW = 1;
        op.sN = C; op.sH = C; op.sW = C;
        unsigned nout = 0;
        int rc = ld.linear_weights({name}, C, op, &nout);
        if (rc) return rc;
        if ((int)nout != K) { set_error("'%s': expected %d outputs, container has %u", name.c_str(), K, nout); return STRAIT_E_FORMAT; }
        op.info.macs_per_sample = (int64_t)C * K;
        op.info.bytes_per_sample = 2LL * C + 2LL * K;
        op.info.gemm_m_per_sample = 1; op.info.gemm_n = K; op.info.gemm_k = C;
        m.ops.push_back(op);
        return 0;
    }

    // a linear layer applied to every row of a [rows][K] activation per sample (token-wise GEMM); several weight
    // matrices of the container may be stacked along the output axis (Q | K | V)
    int token_gemm(const std::string& name, std::initializer_list<std::string> ws, int rows, int in, int K, int N, int act,
                   int res, int out) {
        Op op;
        name_op(op, name, 0);
        op.kind = OP_CONV;
        op.in = in; op.out = out; op.res = res; op.act = act;
        op.P = rows; op.Q = 1; op.H = rows; op.W = 1;
        op.C = K; op.K = N; op.vC = K; op.vR = op.vS = 1; op.vH = op.vW = 1;
        op.sN = K; op.sH = K; op.sW = K;
        unsigned nout = 0;
        int rc = ld.linear_weights(ws, K, op, &nout);
        if (rc) return rc;
        if ((int)nout != N) { set_error("'%s': expected %d outputs, container has %u", name.c_str(), N, nout); return STRAIT_E_FORMAT; }
        op.info.macs_per_sample = (int64_t)rows * K * N;
        op.info.bytes_per_sample = 2LL * rows * ((int64_t)K + (int64_t)N * (res != SLOT_NONE ? 2 : 1));
        op.info.gemm_m_per_sample = rows; op.info.gemm_n = N; op.info.gemm_k = K;
        m.ops.push_back(op);
        return 0;
    }

    // LayerNorm over `width` features of `rows` rows per sample; in_stride: elements between input rows (0 = width)
    int layer_norm(const std::string& name, int in, int out, int out_ref, int rows, int width, float eps, long long in_stride) {
        Op op;
        name_op(op, name, 4);
        op.kind = OP_LAYERNORM;
        op.in = in; op.out = out; op.out_ref = out_ref; op.P = rows; op.K = width; op.eps = eps; op.in_row_stride = in_stride;
        int rc;
        if ((rc = ld.vector_f32(name + ".g", width, &op.bias))) return rc;
        if ((rc = ld.vector_f32(name + ".b", width, &op.beta))) return rc;
        op.info.bytes_per_sample = 4LL * rows * width;
        op.info.weight_bytes = 8LL * width;
        m.ops.push_back(op);
        return 0;
    }

    void attention(const std::string& name, int qkv, int out, int seq, int heads, int hidden) {
        Op op;
        name_op(op, name, 5);
        op.kind = OP_ATTENTION;
        op.in = qkv; op.out = out; op.seq = seq; op.heads = heads; op.P = seq; op.K = hidden;
        op.info.macs_per_sample = 2LL * seq * seq * hidden;
        op.info.bytes_per_sample = 2LL * seq * hidden * 4;
        m.ops.push_back(op);
    }

    // FC on a feature vector f [C] (fp32 logits into the output buffer) -> softmax + top-1
    int head(int f, int C, int classes) {
        Op fc;
        name_op(fc, "fc", 0);
        fc.kind = OP_CONV;
        fc.in = f; fc.out = SLOT_OUT; fc.out_ref = 0; fc.out_f32 = 1;
        fc.C = C; fc.K = classes; fc.vC = C; fc.vR = fc.vS = 1; fc.vH = fc.vW = 1;
        fc.sN = C; fc.sH = C; fc.sW = C;
        unsigned nout = 0;
        int rc = ld.linear_weights({"fc"}, C, fc, &nout);
        if (rc) return rc;
        if ((int)nout != classes) { set_error("fc: expected %d outputs, container has %u", classes, nout); return STRAIT_E_FORMAT; }
        fc.info.macs_per_sample = (int64_t)C * classes;
        fc.info.bytes_per_sample = 2LL * C + 4LL * classes;
        fc.info.gemm_m_per_sample = 1; fc.info.gemm_n = classes; fc.info.gemm_k = C;
        m.ops.push_back(fc);
        pl.put(f);
        Op sm;
        name_op(sm, "softmax", 3);
        sm.kind = OP_SOFTMAX;
        sm.in = SLOT_OUT; sm.out = SLOT_OUT; sm.out_ref = 1; sm.out_ref2 = 2; sm.K = classes;
        sm.info.bytes_per_sample = 8LL * classes + 4;
        m.ops.push_back(sm);
        return 0;
    }
};

static int plan_tiny_cnn(Model& m, Builder& b) {
    const int H = m.hyper[0], W = m.hyper[1], C = m.hyper[2], classes = m.hyper[3];
    int cur, P, Q, rc;
    if ((rc = b.stem("conv0", false, H, W, C, 16, 3, 1, 1, ACT_RELU, 0, &cur, &P, &Q))) return rc;
    int cin = 16;
    const int couts[2] = {32, 64};
    for (int i = 0; i < 2; ++i) {
        const int o = b.pl.get((size_t)b.osz(P, 3, 2, 1) * b.osz(Q, 3, 2, 1) * couts[i]);
        char nm[16];
        snprintf(nm, sizeof(nm), "conv%d", i + 1);
        if ((rc = b.conv(nm, false, cur, P, Q, cin, couts[i], 3, 2, 1, ACT_RELU, SLOT_NONE, o, &P, &Q))) return rc;
        b.pl.put(cur);
        cur = o; cin = couts[i];
    }
    return b.classifier(cur, P, Q, cin, classes);
}

static int plan_resnet50(Model& m, Builder& b) {
    const int H = m.hyper[0], W = m.hyper[1], C = m.hyper[2], classes = m.hyper[3];
    int cur, P, Q, rc;
    if (C == 3 && W % 2 == 0) {
        // one launch reads the image and writes the pooled feature map (the layer carries the pooling's name: that is
        // the activation it produces)
        if ((rc = b.stem_pool("maxpool", true, H, W, &cur, &P, &Q))) return rc;
    } else {
        if ((rc = b.stem("stem", true, H, W, C, 64, 7, 2, 3, ACT_RELU, 0, &cur, &P, &Q))) return rc;
        const int P2 = b.osz(P, 3, 2, 1), Q2 = b.osz(Q, 3, 2, 1);
        const int o = b.pl.get((size_t)P2 * Q2 * 64);
        b.pool("maxpool", POOL_MAX3X3S2, cur, P, Q, 64, o);
        b.pl.put(cur);
        cur = o; P = P2; Q = Q2;
    }
    int cin = 64;
    const int nblocks[4] = {3, 4, 6, 3}, planes[4] = {64, 128, 256, 512};
    int carry_t1 = -1;                                  // output buffer of the next block's c1 when it may be fused with this block's c3
    for (int si = 0; si < 4; ++si)
        for (int bi = 0; bi < nblocks[si]; ++bi) {
            char pre[16];
            snprintf(pre, sizeof(pre), "s%db%d", si + 1, bi);
            const std::string p(pre);
            const int pln = planes[si], stride = (bi == 0 && si > 0) ? 2 : 1;
            const int P2 = b.osz(P, 3, stride, 1), Q2 = b.osz(Q, 3, stride, 1);
            // The projection shortcut of a stage's first block depends only on the block input, as does
            // c1: it is issued first and runs on the side stream beside c1 and c2; c3 joins.
            int sc = cur, down_idx = -1;
            const int block_in = cur;
            if (bi == 0) {
                sc = b.pl.get((size_t)P2 * Q2 * pln * 4);
                if ((rc = b.conv(p + ".down", true, cur, P, Q, cin, pln * 4, 1, stride, 0, ACT_NONE, SLOT_NONE, sc, nullptr, nullptr))) return rc;
                m.ops.back().side = 1;
                down_idx = (int)m.ops.size() - 1;
            }
            const int t1 = carry_t1 >= 0 ? carry_t1 : b.pl.get((size_t)P * Q * pln);
            carry_t1 = -1;
            if ((rc = b.conv(p + ".c1", true, cur, P, Q, cin, pln, 1, 1, 0, ACT_RELU, SLOT_NONE, t1, nullptr, nullptr))) return rc;
            if (si == 0 && bi == 0 && m.ops[0].kind == OP_STEMPOOL && m.ops[0].out == cur && cin == 64 && pln == 64 && m.ops.back().ldw == 64)
                m.ops[0].stem_next = (int)m.ops.size() - 1;
            const int t2 = b.pl.get((size_t)P2 * Q2 * pln);
            if ((rc = b.conv(p + ".c2", true, t1, P, Q, pln, pln, 3, stride, 1, ACT_RELU, SLOT_NONE, t2, nullptr, nullptr))) return rc;
            b.pl.put(t1);
            // a projection that may join the closing convolution's launch reads the block input there: keep it until then
            const bool next_same = bi != nblocks[si] - 1;
            const bool proj = bi == 0 && stride == 1 && next_same && pointwise_pair_proj_supported(pln, cin, pln * 4, pln);
            // elsewhere (stride 2) the closing convolution alone can absorb it, as a second source of its reduction
            const bool proj_conv = bi == 0 && !proj && pln % 64 == 0 && cin % 64 == 0;
            if (bi == 0 && !proj && !proj_conv) b.pl.put(cur);
            const int o = b.pl.get((size_t)P2 * Q2 * pln * 4);
            if ((rc = b.conv(p + ".c3", true, t2, P2, Q2, pln, pln * 4, 1, 1, 0, ACT_RELU, sc, o, nullptr, nullptr))) return rc;
            if (bi == 0) m.ops.back().join = 1;
            // This c3 and the next block's c1 can run as one launch.  That launch writes the c1 output while other
            // workgroups still read this block's c2 output and shortcut, so its buffer is taken before those two are
            // released (it must not reuse them).  The next block's projection shortcut, if any, sits between the two ops.
            const bool last = si == 3 && bi == nblocks[si] - 1;
            const int next_pln = bi == nblocks[si] - 1 ? (si < 3 ? planes[si + 1] : 0) : pln;
            if (!last && pointwise_pair_supported(pln, pln * 4, next_pln) && m.ops.back().ldw == pln) {
                carry_t1 = b.pl.get((size_t)P2 * Q2 * next_pln);
                m.ops.back().pair = bi == nblocks[si] - 1 ? 2 : 1;
                if (proj) {
                    Op& c3 = m.ops.back();
                    if ((rc = b.ld.proj_pair_weights(p + ".c3", pln, p + ".down", cin, pln * 4, c3))) return rc;
                    c3.proj_down = down_idx;
                    m.ops[down_idx].proj_of = (int)m.ops.size() - 1;
                }
            }
            if (proj_conv) {
                Op& c3 = m.ops.back();
                if ((rc = b.ld.proj_pair_weights(p + ".c3", pln, p + ".down", cin, pln * 4, c3))) return rc;
                c3.proj_down = down_idx;
                m.ops[down_idx].proj_of = (int)m.ops.size() - 1;
            }
            if (proj || proj_conv) b.pl.put(block_in);
            b.pl.put(t2);
            b.pl.put(sc);
            cur = o; cin = pln * 4; P = P2; Q = Q2;
        }
    return b.classifier(cur, P, Q, cin, classes);
}

static int plan_mobilenet_v2(Model& m, Builder& b) {
    const int H = m.hyper[0], W = m.hyper[1], C = m.hyper[2], classes = m.hyper[3];
    int cur, P, Q, rc;
    if ((rc = b.stem("stem", true, H, W, C, 32, 3, 2, 1, ACT_RELU6, 0, &cur, &P, &Q))) return rc;
    static const int cfg[7][4] = {{1, 16, 1, 1}, {6, 24, 2, 2}, {6, 32, 3, 2}, {6, 64, 4, 2}, {6, 96, 3, 1}, {6, 160, 3, 2}, {6, 320, 1, 1}};
    int cin = 32, idx = 0;
    for (int g = 0; g < 7; ++g)
        for (int i = 0; i < cfg[g][2]; ++i, ++idx) {
            const int t = cfg[g][0], cout = cfg[g][1], stride = i == 0 ? cfg[g][3] : 1;
            const int hid = cin * t;
            char pre[16];
            snprintf(pre, sizeof(pre), "b%d", idx);
            const std::string p(pre);
            int a = cur;
            if (t != 1) {
                a = b.pl.get((size_t)P * Q * hid);
                if ((rc = b.conv(p + ".expand", true, cur, P, Q, cin, hid, 1, 1, 0, ACT_RELU6, SLOT_NONE, a, nullptr, nullptr))) return rc;
            }
            const int P2 = b.osz(P, 3, stride, 1), Q2 = b.osz(Q, 3, stride, 1);
            const int d = b.pl.get((size_t)P2 * Q2 * hid);
            int Pd, Qd;
            if ((rc = b.dwconv(p + ".dw", a, P, Q, hid, stride, d, &Pd, &Qd))) return rc;
            if (t != 1 && expand_dw_supported(cin, hid, stride)) m.ops[m.ops.size() - 2].dw_next = true;
            // the first block has no expansion: its depthwise layer reads the stem's output, and the two can be one launch
            if (t == 1 && idx == 0 && stride == 1 && hid == 32 && m.ops.size() >= 2 && m.ops[m.ops.size() - 2].kind == OP_STEM3)
                m.ops[m.ops.size() - 2].dw_next = true;
            if (a != cur) b.pl.put(a);
            const bool residual = stride == 1 && cin == cout;
            const int o = b.pl.get((size_t)P2 * Q2 * cout);
            if ((rc = b.conv(p + ".project", true, d, P2, Q2, hid, cout, 1, 1, 0, ACT_NONE, residual ? cur : SLOT_NONE, o, nullptr, nullptr))) return rc;
            b.pl.put(d);
            b.pl.put(cur);
            cur = o; cin = cout; P = P2; Q = Q2;
        }
    const int hd = b.pl.get((size_t)P * Q * 1280);
    if ((rc = b.conv("head", true, cur, P, Q, cin, 1280, 1, 1, 0, ACT_RELU6, SLOT_NONE, hd, nullptr, nullptr))) return rc;
    b.pl.put(cur);
    return b.classifier(hd, P, Q, 1280, classes);
}

// VGG-19: 3x3 convolutions with bias and ReLU, 2x2 max pooling after the 2nd, 4th, 8th, 12th and 16th, then three
// fully connected layers.  The first of them reads the last feature map flattened channel-major in the
// container; its weight [out, C, h, w] is re-laid like a convolution's to [out][h][w][C], which is the order the
// NHWC feature map already has in memory, so the layer is a plain matrix product over h*w*C inputs.
static int plan_vgg19(Model& m, Builder& b) {
    const int H = m.hyper[0], W = m.hyper[1], C = m.hyper[2], classes = m.hyper[3], fcw = m.hyper[4];
    if (H % 32 != 0 || W % 32 != 0 || fcw <= 0 || fcw % 8 != 0) { set_error("VGG-19: H and W must be multiples of 32 and the FC width a multiple of 8"); return STRAIT_E_SHAPE; }
    static const int cfg[21] = {64, 64, 0, 128, 128, 0, 256, 256, 256, 256, 0, 512, 512, 512, 512, 0, 512, 512, 512, 512, 0};
    int cur = SLOT_NONE, P = H, Q = W, cin = C, idx = 0, rc;
    for (int i = 0; i < 21; ++i) {
        char nm[16];
        if (cfg[i] == 0) {
            const int o = b.pl.get((size_t)(P / 2) * (Q / 2) * cin);
            snprintf(nm, sizeof(nm), "pool%d", idx);
            b.pool(nm, POOL_MAX2X2S2, cur, P, Q, cin, o);
            b.pl.put(cur);
            cur = o; P /= 2; Q /= 2;
            continue;
        }
        snprintf(nm, sizeof(nm), "conv%d", idx);
        if (idx == 0) {
            if ((rc = b.stem(nm, false, H, W, C, cfg[i], 3, 1, 1, ACT_RELU, 0, &cur, &P, &Q))) return rc;
        } else {
            const int o = b.pl.get((size_t)P * Q * cfg[i]);
            if ((rc = b.conv(nm, false, cur, P, Q, cin, cfg[i], 3, 1, 1, ACT_RELU, SLOT_NONE, o, nullptr, nullptr))) return rc;
            b.pl.put(cur);
            cur = o;
        }
        cin = cfg[i];
        ++idx;
    }
    // fc1: a P x Q "convolution" without padding on the P x Q feature map = one output position
    const int f1 = b.pl.get(fcw);
    {
        Op op;
        name_op(op, "fc1", 0);
        op.kind = OP_CONV;
        op.in = cur; op.out = f1; op.act = ACT_RELU;
        const int Cin = P * Q * cin;
        op.C = Cin; op.K = fcw; op.vC = Cin; op.vR = op.vS = 1; op.vH = op.vW = 1;
        op.sN = Cin; op.sH = Cin; op.sW = Cin;
        if ((rc = b.ld.conv_weights("fc1", false, fcw, cin, P, Q, op))) return rc;
        op.info.macs_per_sample = (int64_t)Cin * fcw;
        op.info.bytes_per_sample = 2LL * Cin + 2LL * fcw;
        op.info.gemm_m_per_sample = 1; op.info.gemm_n = fcw; op.info.gemm_k = Cin;
        m.ops.push_back(op);
    }
    b.pl.put(cur);
    const int f2 = b.pl.get(fcw);
    if ((rc = b.dense("fc2", f1, fcw, fcw, ACT_RELU, f2))) return rc;
    b.pl.put(f1);
    rc = b.head(f2, fcw, classes);
    return rc;
}

// Vision Transformer with 16x16 patches, pre-LayerNorm blocks:
//   tokens = [cls ; patches W_p + b_p] + pos;  z += Attn(LN1(z)) W_o + b_o;  z += GELU(LN2(z) W_1 + b_1) W_2 + b_2;
//   logits = LN(z)[token 0] W_h + b_h.
// The patch embedding is a 16x16 convolution of stride 16 (the stem path: its row taps are contiguous in memory);
// every sequence has the same length, so the attention kernel's valid lengths are all S.
static int plan_vit(Model& m, Builder& b) {
    const int H = m.hyper[0], W = m.hyper[1], C = m.hyper[2], classes = m.hyper[3];
    const int layers = m.hyper[4], hidden = m.hyper[5], heads = m.hyper[6], ffn = m.hyper[7];
    if (H % 16 != 0 || W % 16 != 0) { set_error("ViT: H and W must be multiples of the 16-pixel patch"); return STRAIT_E_SHAPE; }
    if (layers <= 0 || heads <= 0 || hidden != heads * 64) { set_error("ViT: head dimension must be 64 (hidden %d, heads %d)", hidden, heads); return STRAIT_E_SHAPE; }
    if (ffn <= 0 || ffn % 8 != 0) { set_error("ViT: ffn width must be a multiple of 8"); return STRAIT_E_SHAPE; }
    const int T = (H / 16) * (W / 16), seq = T + 1;
    if (seq > 256) { set_error("ViT: %d tokens, at most 256 are supported", seq); return STRAIT_E_SHAPE; }
    m.seq = seq; m.hidden = hidden;
    Loader& ld = b.ld;
    auto gemm = [&](const std::string& name, std::initializer_list<std::string> ws, int in, int K, int N, int act, int res, int out) {
        return b.token_gemm(name, ws, seq, in, K, N, act, res, out);
    };
    auto lnorm = [&](const std::string& name, int in, int out, int rows, long long in_stride) {
        return b.layer_norm(name, in, out, 0, rows, hidden, 1e-6f, in_stride);
    };
    int patches, P, Q, rc;
    if ((rc = b.stem("patch", false, H, W, C, hidden, 16, 16, 0, ACT_NONE, 0, &patches, &P, &Q))) return rc;
    const size_t tok = (size_t)seq * hidden;
    int z = b.pl.get(tok);
    {
        Op op;
        name_op(op, "tokens", 6);
        op.kind = OP_TOKENS;
        op.in = patches; op.out = z; op.P = seq; op.K = hidden;     // P: rows written per sample (T patches + the class token)
        if ((rc = ld.vector_f32("cls", hidden, &op.bias))) return rc;
        const TensorView* pos = ld.c.find("pos");
        if (!pos || pos->ndim != 2 || pos->shape[0] != (unsigned)seq || pos->shape[1] != (unsigned)hidden) { set_error("'pos': expected [%d,%d]", seq, hidden); return STRAIT_E_FORMAT; }
        std::vector<float> f(pos->count);
        for (size_t i = 0; i < pos->count; ++i) f[i] = (float)pos->data[i];
        void* d = nullptr;
        if ((rc = ld.upload(f.data(), f.size() * 4, &d))) return rc;
        op.beta = (const float*)d;
        op.info.bytes_per_sample = 2LL * ((int64_t)T * hidden + (int64_t)seq * hidden);
        op.info.weight_bytes = 4LL * (seq + 1) * hidden;
        m.ops.push_back(op);
    }
    b.pl.put(patches);
    for (int i = 0; i < layers; ++i) {
        char pre[16];
        snprintf(pre, sizeof(pre), "l%d", i);
        const std::string p(pre);
        const int n1 = b.pl.get(tok);
        if ((rc = lnorm(p + ".ln1", z, n1, seq, 0))) return rc;
        const int qkv = b.pl.get(3 * tok);
        if ((rc = gemm(p + ".qkv", {p + ".q", p + ".k", p + ".v"}, n1, hidden, 3 * hidden, ACT_NONE, SLOT_NONE, qkv))) return rc;
        b.pl.put(n1);
        const int att = b.pl.get(tok);
        b.attention(p + ".attn", qkv, att, seq, heads, hidden);
        b.pl.put(qkv);
        const int z1 = b.pl.get(tok);
        if ((rc = gemm(p + ".o", {p + ".o"}, att, hidden, hidden, ACT_NONE, z, z1))) return rc;
        b.pl.put(att);
        b.pl.put(z);
        const int n2 = b.pl.get(tok);
        if ((rc = lnorm(p + ".ln2", z1, n2, seq, 0))) return rc;
        const int f = b.pl.get((size_t)seq * ffn);
        if ((rc = gemm(p + ".ffn1", {p + ".ffn1"}, n2, hidden, ffn, ACT_GELU, SLOT_NONE, f))) return rc;
        b.pl.put(n2);
        const int z2 = b.pl.get(tok);
        if ((rc = gemm(p + ".ffn2", {p + ".ffn2"}, f, ffn, hidden, ACT_NONE, z1, z2))) return rc;
        b.pl.put(f);
        b.pl.put(z1);
        z = z2;
    }
    // the head reads token 0 only: the closing LayerNorm runs on that row of every sample
    const int feat = b.pl.get(hidden);
    if ((rc = lnorm("ln", z, feat, 1, (long long)seq * hidden))) return rc;
    b.pl.put(z);
    return b.head(feat, hidden, classes);
}

static int plan_encoder(Model& m, Builder& b) {
    const int layers = m.hyper[0], hidden = m.hyper[1], heads = m.hyper[2], ffn = m.hyper[3], seq = m.hyper[4];
    if (heads <= 0 || hidden != heads * 64) { set_error("encoder: head dimension must be 64 (hidden %d, heads %d)", hidden, heads); return STRAIT_E_SHAPE; }
    if (seq <= 0 || seq > 256) { set_error("encoder: sequence length %d must be in 1..256", seq); return STRAIT_E_SHAPE; }
    if (ffn % 8 != 0) { set_error("encoder: ffn width must be a multiple of 8"); return STRAIT_E_SHAPE; }
    auto gemm = [&](const std::string& name, std::initializer_list<std::string> ws, int in, int K, int N, int act, int res, int out) {
        return b.token_gemm(name, ws, seq, in, K, N, act, res, out);
    };
    auto lnorm = [&](const std::string& name, int in, int out, int out_ref) {
        return b.layer_norm(name, in, out, out_ref, seq, hidden, 1e-12f, 0);
    };
    int x = SLOT_INPUT, rc;
    const size_t tok = (size_t)seq * hidden;
    for (int i = 0; i < layers; ++i) {
        char pre[16];
        snprintf(pre, sizeof(pre), "l%d", i);
        const std::string p(pre);
        const int qkv = b.pl.get(3 * tok);
        if ((rc = gemm(p + ".qkv", {p + ".q", p + ".k", p + ".v"}, x, hidden, 3 * hidden, ACT_NONE, SLOT_NONE, qkv))) return rc;
        const int att = b.pl.get(tok);
        b.attention(p + ".attn", qkv, att, seq, heads, hidden);
        b.pl.put(qkv);
        const int t = b.pl.get(tok);
        if ((rc = gemm(p + ".o", {p + ".o"}, att, hidden, hidden, ACT_NONE, x, t))) return rc;
        b.pl.put(att);
        const int h = b.pl.get(tok);
        if ((rc = lnorm(p + ".ln1", t, h, 0))) return rc;
        b.pl.put(t);
        b.pl.put(x);
        const int f = b.pl.get((size_t)seq * ffn);
        if ((rc = gemm(p + ".ffn1", {p + ".ffn1"}, h, hidden, ffn, ACT_GELU, SLOT_NONE, f))) return rc;
        const int t2 = b.pl.get(tok);
        if ((rc = gemm(p + ".ffn2", {p + ".ffn2"}, f, ffn, hidden, ACT_NONE, h, t2))) return rc;
        b.pl.put(f);
        const bool last = i == layers - 1;
        const int y = last ? SLOT_OUT : b.pl.get(tok);
        if ((rc = lnorm(p + ".ln2", t2, y, 0))) return rc;
        b.pl.put(t2);
        b.pl.put(h);
        x = y;
    }
    Op am;
    name_op(am, "argmax", 2);
    am.kind = OP_POOL; am.sub = POOL_ARGMAX;
    am.in = SLOT_OUT; am.out = SLOT_OUT; am.out_ref = 3; am.K = hidden; am.P = seq;
    am.info.bytes_per_sample = 2LL * hidden + 4;
    m.ops.push_back(am);
    return 0;
}

size_t Model::out_bytes(int b) const {
    if (arch == STRAIT_ARCH_ENCODER) return (size_t)b * seq * hidden * 2 + (size_t)b * 4;
    return (size_t)b * classes * 8 + (size_t)b * 4;
}
size_t Model::out_offset(int ref, int b) const {
    switch (ref) {
        case 1: return (size_t)b * classes * 4;
        case 2: return (size_t)b * classes * 8;
        case 3: return (size_t)b * seq * hidden * 2;
        default: return 0;
    }
}

int build_plan(Model& m, const void* blob, size_t bytes) {
    Container c;
    int rc = parse_container(blob, bytes, c);
    if (rc) return rc;
    m.arch = c.arch;
    for (int i = 0; i < 8; ++i) m.hyper[i] = (int)c.hyper[i];
    Loader ld{m, c};
    Builder b{m, ld, Planner{m, {}}};
    switch (m.arch) {
        case STRAIT_ARCH_TINY_CNN:
        case STRAIT_ARCH_RESNET50:
        case STRAIT_ARCH_MOBILENETV2:
            if (m.hyper[0] <= 0 || m.hyper[1] <= 0 || m.hyper[2] <= 0 || m.hyper[2] > 4 || m.hyper[3] <= 0 || m.hyper[0] > 4096 || m.hyper[1] > 4096) {
                set_error("CNN hyper-parameters out of range (H %d, W %d, C %d, classes %d)", m.hyper[0], m.hyper[1], m.hyper[2], m.hyper[3]);
                return STRAIT_E_SHAPE;
            }
            m.in_elems = (size_t)m.hyper[0] * m.hyper[1] * m.hyper[2];
            m.classes = m.hyper[3];
            rc = m.arch == STRAIT_ARCH_TINY_CNN ? plan_tiny_cnn(m, b) : m.arch == STRAIT_ARCH_RESNET50 ? plan_resnet50(m, b) : plan_mobilenet_v2(m, b);
            break;
        case STRAIT_ARCH_VGG19:
        case STRAIT_ARCH_VIT:
            if (m.hyper[0] <= 0 || m.hyper[1] <= 0 || m.hyper[2] != 3 || m.hyper[3] <= 0 || m.hyper[0] > 4096 || m.hyper[1] > 4096) {
                set_error("image model hyper-parameters out of range (H %d, W %d, C %d, classes %d)", m.hyper[0], m.hyper[1], m.hyper[2], m.hyper[3]);
                return STRAIT_E_SHAPE;
            }
            m.in_elems = (size_t)m.hyper[0] * m.hyper[1] * m.hyper[2];
            m.classes = m.hyper[3];
            rc = m.arch == STRAIT_ARCH_VGG19 ? plan_vgg19(m, b) : plan_vit(m, b);
            break;
        case STRAIT_ARCH_ENCODER:
            if (m.hyper[0] <= 0 || m.hyper[1] <= 0 || m.hyper[3] <= 0) { set_error("encoder hyper-parameters out of range"); return STRAIT_E_SHAPE; }
            m.seq = m.hyper[4]; m.hidden = m.hyper[1];
            m.in_elems = (size_t)m.seq * m.hidden;
            rc = plan_encoder(m, b);
            break;
        default:
            set_error("unknown architecture id %d", m.arch);
            return STRAIT_E_FORMAT;
    }
    return rc;
}

// ------------------------------------------------------------------------------------------
static void* slot_ptr(Model& m, Instance& in, int slot, int ref, int batch) {
    if (slot == SLOT_INPUT) return in.dev_in;
    if (slot == SLOT_OUT) return (char*)in.dev_out + m.out_offset(ref, batch);
    if (slot >= 0) return in.bufs[slot];
    return nullptr;
}

int run_plan(Model& m, Instance& in, int batch, hipStream_t stream, int hp, int last_layer, bool timed, int first_layer) {
    const int n = (int)m.ops.size();
    if (last_layer < 0 || last_layer >= n) last_layer = n - 1;
    // Per-layer timing and prefix runs keep everything on the one stream (their events bracket single launches).
    if (first_layer < 0 || first_layer > last_layer) first_layer = 0;
    const bool branches = !timed && first_layer == 0 && last_layer == n - 1 && in.side != nullptr && m.ctx->branch_streams;
    bool forked = false;
    hipStream_t main_stream = stream;
    if (timed) in.layer_skipped.assign(m.ops.size(), 0);
    int fused_away = -1;                                // op already computed by the pair launch of an earlier op
    int stem_next_done = -1;                            // the 1x1 convolution already computed inside the fused stem
    // whether op i (a block-closing pointwise convolution) runs as one launch with the op `pair` further on, and whether
    // that launch also absorbs the block's projection shortcut; the projection op asks the same question about its block
    auto pair_here = [&](int i) {
        const Op& op = m.ops[i];
        if (i > last_layer || m.ctx->pair_min_pixels <= 0) return 0;
        const long long pixels = (long long)batch * op.P * op.Q;
        const bool with_proj = op.w_proj && pixels >= m.ctx->proj_min_pixels;
        if (op.pair && i + op.pair <= last_layer) {
            if (with_proj && pointwise_pair_proj_supported(op.vC, m.ops[op.proj_down].vC, op.K, m.ops[i + op.pair].K)) return 2;
            if (pixels >= m.ctx->pair_min_pixels) return 1;
        }
        return with_proj ? 3 : 0;                       // 3: no pair, but the convolution takes the projection as a second source
    };
    for (int i = first_layer; i <= last_layer; ++i) {
        const Op& op = m.ops[i];
        stream = main_stream;
        if (i == fused_away || i == stem_next_done || (op.proj_of >= 0 && pair_here(op.proj_of) >= 2)) {
            if (timed) { HIP_TRY(hipEventRecord(in.layer_ev[i], stream)); in.layer_skipped[i] = 1; }
            continue;
        }
        // a branch pays a fork and a join (two event hand-overs between streams): only worth it for a launch
        // of some size; smaller ones stay in line, where they may also split their reduction
        if (branches && op.side && (long long)batch * op.P * op.Q * op.K >= 8000000LL) {
            HIP_TRY(hipEventRecord(in.ev_fork, main_stream));
            HIP_TRY(hipStreamWaitEvent(in.side, in.ev_fork, 0));
            stream = in.side;
            forked = true;
        }
        if (branches && op.join && forked) {
            HIP_TRY(hipEventRecord(in.ev_join, in.side));
            HIP_TRY(hipStreamWaitEvent(main_stream, in.ev_join, 0));
            forked = false;
        }
        if (timed) HIP_TRY(hipEventRecord(in.layer_ev[i], stream));
        const void* src = slot_ptr(m, in, op.in, 0, batch);
        void* dst = slot_ptr(m, in, op.out, op.out_ref, batch);
        int rc = 0;
        switch (op.kind) {
            case OP_CONV: {
                // An inverted residual block's expansion and depthwise layer as one launch, the expanded tensor staying in
                // LDS.  It pays where launches are what a batch costs (MobileNetV2 up to batch 8: -3.5 to -7 % per batch) and
                // on the one layer whose expanded tensor dwarfs its input and output while two workgroups still fit a compute
                // unit (112 x 112 x 16 -> 96 at stride 2: -10 % per batch of 64 or 128); elsewhere the two launches, each
                // with every lane busy, are as fast or faster (all blocks fused at batch 64: +3 %).
                if (op.dw_next && i + 1 <= last_layer && m.ctx->pair_min_pixels > 0 &&
                    (batch <= 8 || (m.ops[i + 1].stride == 2 && op.vC <= 16 && (long long)batch * op.P * op.Q * op.K >= 36000000LL))) {
                    const Op& dw = m.ops[i + 1];
                    rc = launch_expand_dw((const half_t*)src, batch, op.P, op.Q, op.vC, op.w, op.ldw, op.bias, op.K, op.act, dw.w, dw.bias,
                                          dw.stride, dw.act, (half_t*)slot_ptr(m, in, dw.out, dw.out_ref, batch), hp, stream);
                    fused_away = i + 1;
                    break;
                }
                const int how = pair_here(i);
                if (how == 1 || how == 2) {
                    const Op& nx = m.ops[i + op.pair];
                    PairParams q{};
                    q.x = (const half_t*)src;
                    if (how == 2) {
                        q.x2 = (const half_t*)slot_ptr(m, in, m.ops[op.proj_down].in, 0, batch);
                        q.K2 = m.ops[op.proj_down].vC;
                        q.w3 = op.w_proj; q.b3 = op.bias_proj;
                    } else {
                        q.w3 = op.w; q.b3 = op.bias;
                        q.res = (const half_t*)slot_ptr(m, in, op.res, 0, batch);
                    }
                    q.y = (half_t*)dst;
                    q.w1 = nx.w; q.b1 = nx.bias; q.z = (half_t*)slot_ptr(m, in, nx.out, nx.out_ref, batch);
                    q.M = batch * op.P * op.Q; q.K1 = op.vC; q.N1 = op.K; q.N2 = nx.K; q.act1 = op.act; q.act2 = nx.act; q.hp = hp;
                    rc = launch_pointwise_pair(q, stream);
                    fused_away = i + op.pair;
                    break;
                }
                ConvParams p{};
                p.x = (const half_t*)src; p.w = op.w; p.bias = op.bias;
                p.res = (const half_t*)slot_ptr(m, in, op.res, 0, batch);
                p.y = dst;
                p.M = batch * op.P * op.Q; p.PQ = op.P * op.Q; p.Q = op.Q;
                p.H = op.vH; p.W = op.vW; p.C = op.vC; p.R = op.vR; p.S = op.vS;
                p.stride_h = op.stride; p.stride_w = op.stride_w; p.pad_h = op.pad_h; p.pad_w = op.pad_w;
                p.sN = op.sN; p.sH = op.sH; p.sW = op.sW;
                p.Kg = op.vR * op.vS * op.vC; p.ldw = op.ldw;
                p.Cout = op.K; p.ldy = op.K; p.act = op.act; p.out_f32 = op.out_f32; p.hp = hp;
                if (how == 3) {
                    const Op& dn = m.ops[op.proj_down];
                    p.w = op.w_proj; p.bias = op.bias_proj; p.res = nullptr;
                    p.x2 = (const half_t*)slot_ptr(m, in, dn.in, 0, batch);
                    p.K2 = dn.vC; p.stride2 = dn.stride; p.sH2 = dn.sH; p.sW2 = dn.sW; p.sN2 = dn.sN;
                    p.Kg = op.vC + dn.vC; p.ldw = p.Kg;
                }
                // the split-K workspace belongs to the main stream's launches; a branch running beside them goes without
                if (stream == main_stream) { p.ws = in.splitk_ws; p.ws_bytes = SPLITK_WS_BYTES; }
                rc = launch_conv(p, stream);
                break;
            }
            case OP_STEMPOOL:
                if (op.stem_next >= 0 && op.stem_next <= last_layer && m.ctx->pair_min_pixels > 0) {
                    const Op& c1 = m.ops[op.stem_next];
                    rc = launch_stem_pool((const half_t*)src, op.w, op.bias, batch, op.H, op.W, (half_t*)dst, hp, stream, c1.w, c1.bias,
                                          (half_t*)slot_ptr(m, in, c1.out, c1.out_ref, batch));
                    stem_next_done = op.stem_next;
                    break;
                }
                rc = launch_stem_pool((const half_t*)src, op.w, op.bias, batch, op.H, op.W, (half_t*)dst, hp, stream);
                break;
            case OP_STEM3:
                if (op.dw_next && i + 1 <= last_layer && m.ctx->pair_min_pixels > 0) {
                    // with the first block's depthwise layer behind it in the same launch: the stem's output stays in LDS
                    const Op& dw = m.ops[i + 1];
                    rc = launch_stem3x3s2_dw((const half_t*)src, op.w, op.bias, op.act, dw.w, dw.bias, dw.act, batch, op.H, op.W,
                                             (half_t*)slot_ptr(m, in, dw.out, dw.out_ref, batch), hp, stream);
                    fused_away = i + 1;
                    break;
                }
                rc = launch_stem3x3s2((const half_t*)src, op.w, op.bias, batch, op.H, op.W, op.K, op.act, (half_t*)dst, hp, stream);
                break;
            case OP_PACK:
                rc = launch_pack_input((const half_t*)src, batch, op.H, op.W, op.C, (half_t*)dst, op.Hp, op.Wp, op.Cpad, op.pad, op.pad, hp, stream);
                break;
            case OP_DWCONV:
                rc = launch_dwconv3x3((const half_t*)src, batch, op.H, op.W, op.C, op.w, op.bias, op.stride, op.act, (half_t*)dst, hp, stream);
                break;
            case OP_POOL:
                if (op.sub == POOL_MAX3X3S2) rc = launch_maxpool3x3s2((const half_t*)src, batch, op.H, op.W, op.C, (half_t*)dst, hp, stream);
                else if (op.sub == POOL_MAX2X2S2) rc = launch_maxpool2x2s2((const half_t*)src, batch, op.H, op.W, op.C, (half_t*)dst, hp, stream);
                else if (op.sub == POOL_GLOBAL_AVG) rc = launch_global_avgpool((const half_t*)src, batch, op.H * op.W, op.C, (half_t*)dst, hp, stream);
                else rc = launch_argmax_f16((const half_t*)src, batch, op.K, (long long)op.P * op.K, (int32_t*)dst, hp, stream);
                break;
            case OP_SOFTMAX:
                rc = launch_softmax_top1((const float*)src, batch, op.K, (float*)dst, (int32_t*)slot_ptr(m, in, SLOT_OUT, op.out_ref2, batch), hp, stream);
                break;
            case OP_LAYERNORM:
                rc = launch_layernorm((const half_t*)src, op.bias, op.beta, batch * op.P, op.K, op.eps, (half_t*)dst, hp, stream, op.in_row_stride);
                break;
            case OP_TOKENS:
                rc = launch_vit_tokens((const half_t*)src, op.bias, op.beta, batch, op.P - 1, op.K, (half_t*)dst, hp, stream);
                break;
            case OP_ATTENTION:
                rc = launch_attention((const half_t*)src, in.dev_valid, batch, op.seq, op.heads, (half_t*)dst, hp, stream);
                break;
            default:
                set_error("unknown op kind %d", op.kind);
                rc = STRAIT_E_INVALID;
        }
        if (rc) {
            if (forked) { (void)hipEventRecord(in.ev_join, in.side); (void)hipStreamWaitEvent(main_stream, in.ev_join, 0); }
            return rc;
        }
    }
    if (forked) {                                       // a branch nobody joined: the main stream still waits for it
        HIP_TRY(hipEventRecord(in.ev_join, in.side));
        HIP_TRY(hipStreamWaitEvent(main_stream, in.ev_join, 0));
    }
    if (timed) HIP_TRY(hipEventRecord(in.layer_ev[last_layer + 1], main_stream));
    return 0;
}

}  // namespace strait
