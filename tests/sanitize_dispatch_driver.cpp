// Driver for tests/test_dispatch_sanitizers.py: the library's host side (csrc/msla_api.cpp: argument
// checks, workspace carving, launch order) built for the CPU with AddressSanitizer + UBSan and linked
// against the launcher stand-ins below instead of the GPU kernels.  A stand-in launches nothing: it checks
// that every pointer it is handed, with the extent the real kernel would touch, lies inside one of the
// buffers the caller passed to the entry point (x, weights, out, workspace ...), 16-byte aligned -- i.e.
// that the carving of the workspace and the pointer arithmetic of the dispatcher are right for that shape.
// The entry points are then called over a list of shapes, all storage types and all code paths.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <string>
#include <vector>

#include "../include/msla.h"
#include "../paper_2205_14756_amd/csrc/msla_kernels.h"

namespace {

struct Region {
    std::string name;
    const char* base;
    size_t bytes;
};
std::vector<Region> g_regions;
std::string g_case;
int g_failures = 0;
long g_checks = 0;

void fail(const std::string& what) {
    std::fprintf(stderr, "[%s] %s\n", g_case.c_str(), what.c_str());
    ++g_failures;
}

// [p, p + bytes) must lie inside one registered buffer
void inside(const void* p, size_t bytes, const char* what) {
    ++g_checks;
    if (p == nullptr) return fail(std::string(what) + ": null pointer");
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return fail(std::string(what) + ": not 16-byte aligned");
    const char* c = static_cast<const char*>(p);
    for (const Region& r : g_regions)
        if (c >= r.base && c + bytes <= r.base + r.bytes) return;
    char msg[256];
    std::snprintf(msg, sizeof msg, "%s: %zu bytes at %p lie in no buffer of the call", what, bytes, p);
    fail(msg);
}

// the byte ranges handed to one launch must not overlap each other
struct Span {
    const void* p;
    size_t bytes;
    const char* what;
};
void disjoint(std::initializer_list<Span> spans) {
    ++g_checks;
    for (auto a = spans.begin(); a != spans.end(); ++a)
        for (auto b = a + 1; b != spans.end(); ++b) {
            const char *pa = static_cast<const char*>(a->p), *pb = static_cast<const char*>(b->p);
            if (pa && pb && pa < pb + b->bytes && pb < pa + a->bytes) fail(std::string(a->what) + " overlaps " + b->what);
        }
}

size_t esz(int dt) { return dt == 0 ? 4 : 2; }

char* buffer(const char* name, size_t bytes) {
    char* p = static_cast<char*>(std::aligned_alloc(256, (bytes + 255) / 256 * 256 + 256));
    if (!p) { std::fprintf(stderr, "out of memory\n"); std::exit(2); }
    g_regions.push_back({name, p, bytes});
    return p;
}
void release_all() {
    for (const Region& r : g_regions) std::free(const_cast<char*>(r.base));
    g_regions.clear();
}

}  // namespace

// ---------------------------------------------------------------- the HIP runtime calls of the dispatcher
extern "C" {
hipError_t hipGetDevice(int* d) { *d = 0; return hipErrorNoDevice; }
hipError_t hipDeviceGetAttribute(int*, hipDeviceAttribute_t, int) { return hipErrorNoDevice; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind, hipStream_t) {
    inside(dst, bytes, "copy destination");
    inside(src, bytes, "copy source");
    return hipSuccess;
}
}

// ---------------------------------------------------------------- launcher stand-ins
namespace msla {

hipError_t launch_linear(int dt, const void* x, const void* w, void* y, long n, int c_in, int c_out, hipStream_t) {
    inside(x, (size_t)n * c_in * esz(dt), "linear x");
    inside(w, (size_t)c_out * c_in * esz(dt), "linear w");
    inside(y, (size_t)n * c_out * esz(dt), "linear y");
    return hipSuccess;
}
hipError_t launch_linear_act(int dt, const void* x, const void* w, void* y, long n, int c_in, int c_out, int, hipStream_t s) {
    return launch_linear(dt, x, w, y, n, c_in, c_out, s);
}
hipError_t launch_qkv_project(int dt, const void* x, const void* w_qkv, void* q_ms, long q_ms_stride, void* kv_raw,
                              long kv_tok_stride, long kv_head_stride, long kv_span, long n, int c_in, int heads, hipStream_t) {
    const size_t e = esz(dt);
    inside(x, (size_t)n * c_in * e, "projection x");
    inside(w_qkv, (size_t)3 * heads * 16 * c_in * e, "projection w_qkv");
    inside(q_ms, ((size_t)(n - 1) * q_ms_stride + (size_t)heads * 16) * e, "projection raw-Q columns of q_ms");
    inside(kv_raw, (size_t)kv_span * e, "projection K|V map");
    // the last token's last head must end inside the span
    if ((n - 1) * kv_tok_stride + (long)(heads - 1) * kv_head_stride + 32 > kv_span) fail("K|V strides run past the span");
    disjoint({{x, (size_t)n * c_in * e, "projection x"}, {q_ms, (size_t)n * q_ms_stride * e, "q_ms"}, {kv_raw, (size_t)kv_span * e, "K|V map"}});
    return hipSuccess;
}
static void check_aggregate(int dt, const AggregateArgs& a, int d, const char* who) {
    const size_t e = esz(dt);
    const long T = (long)a.B * a.H * a.W;
    const int Ct = a.heads * d;
    std::string w(who);
    inside(a.q, ((size_t)(T - 1) * a.q_ts + (size_t)(a.heads - 1) * a.q_hs + d) * e, (w + " raw Q map").c_str());
    inside(a.k, ((size_t)(T - 1) * a.k_ts + (size_t)(a.heads - 1) * a.k_hs + d) * e, (w + " raw K map").c_str());
    inside(a.v, ((size_t)(T - 1) * a.v_ts + (size_t)(a.heads - 1) * a.v_hs + d) * e, (w + " raw V map").c_str());
    if (a.ks > 0 || a.copy_raw_q) inside(a.q_ms, (size_t)T * a.S * Ct * e, (w + " q_ms").c_str());
    inside(a.partials, (size_t)a.B * a.S * a.heads * a.nchunks * d * (d + 1) * 4, (w + " partial states").c_str());
    if (a.ks > 0) {
        inside(a.w_dw, (size_t)3 * Ct * a.ks * a.ks * e, (w + " w_dw of the scale").c_str());
        inside(a.w_gpw, (size_t)3 * Ct * d * e, (w + " w_gpw of the scale").c_str());
        if (a.branch < 1 || a.branch >= a.S) fail(w + ": branch index out of range");
    }
    if (a.nchunks < 1 || a.tiles_per_chunk < 1) fail(w + ": empty chunking");
    if (a.ks > 0 || a.copy_raw_q)       // (the raw Q map may be the branch-0 columns of q_ms itself: they are only read)
        disjoint({{a.q_ms, (size_t)T * a.S * Ct * e, "q_ms"}, {a.partials, (size_t)a.B * a.S * a.heads * a.nchunks * d * (d + 1) * 4, "partial states"},
                  {a.k, ((size_t)(T - 1) * a.k_ts + (size_t)(a.heads - 1) * a.k_hs + d) * e, "raw K map"}});
}
hipError_t launch_aggregate(int dt, const AggregateArgs& a, hipStream_t) {
    check_aggregate(dt, a, 16, "aggregate");
    if ((long)a.nchunks * a.tiles_per_chunk < (long)((a.H + kAggTileH - 1) / kAggTileH) * ((a.W + kAggTileW - 1) / kAggTileW))
        fail("aggregate: the chunks do not cover the image's tiles");
    return hipSuccess;
}
hipError_t launch_aggregate_mfma(int dt, const AggregateArgs& a, hipStream_t) {
    check_aggregate(dt, a, 16, "aggregate (matrix cores)");
    if ((long)a.nchunks * a.tiles_per_chunk <
        (long)((a.H + kAggMfmaTileH - 1) / kAggMfmaTileH) * ((a.W + kAggMfmaTileW - 1) / kAggMfmaTileW))
        fail("aggregate (matrix cores): the chunks do not cover the image's tiles");
    if (a.ks == 7) return hipErrorNotSupported;     // as the real launcher: the caller falls back
    return hipSuccess;
}
hipError_t launch_aggregate_mfma_pair(int dt, const AggregateArgs& a0, const AggregateArgs& a1, hipStream_t s) {
    if (!((a0.ks == 3 && a1.ks == 5) || (a0.ks == 5 && a1.ks == 3))) return hipErrorNotSupported;
    (void)launch_aggregate_mfma(dt, a0, s);
    (void)launch_aggregate_mfma(dt, a1, s);
    return hipSuccess;
}
hipError_t launch_aggregate32(int dt, const AggregateArgs& a, hipStream_t) {
    check_aggregate(dt, a, 32, "aggregate (heads of 32)");
    return hipSuccess;
}
hipError_t launch_raw_state(int dt, const AggregateArgs& a, hipStream_t) {
    check_aggregate(dt, a, 16, "raw state");
    return hipSuccess;
}
hipError_t launch_state_finalize(int, const float* partials, float* kv32, void* kvfrag, float* kvscale, int n_states, int nchunks,
                                 hipStream_t, int split) {
    inside(partials, (size_t)n_states * nchunks * 272 * 4, "finalize partial states");
    inside(kv32, (size_t)n_states * 272 * 4, "finalize kv32");
    inside(kvfrag, (size_t)n_states * 2048, "finalize operand blocks");
    inside(kvscale, (size_t)n_states * 4, "finalize scales");
    if (split != 0 && split != 8) fail("finalize: split");
    disjoint({{partials, (size_t)n_states * nchunks * 272 * 4, "partial states"}, {kv32, (size_t)n_states * 272 * 4, "kv32"},
              {kvfrag, (size_t)n_states * 2048, "operand blocks"}, {kvscale, (size_t)n_states * 4, "scales"}});
    return hipSuccess;
}
hipError_t launch_pair_head8_weights(int dt, const void* w_qkv, const void* w_dw, const void* w_gpw, void* o_qkv, void* o_dw,
                                     void* o_gpw, int C, int heads8, const int* scales, int n_scales, hipStream_t) {
    const size_t e = esz(dt), rows = (size_t)3 * heads8 * 8;
    size_t dw = 0;
    for (int i = 0; i < n_scales; ++i) dw += rows * scales[i] * scales[i];
    inside(w_qkv, rows * C * e, "pairing: w_qkv");
    inside(o_qkv, rows * C * e, "pairing: rearranged w_qkv");
    if (n_scales > 0) {
        inside(w_dw, dw * e, "pairing: w_dw");
        inside(w_gpw, (size_t)n_scales * rows * 8 * e, "pairing: w_gpw");
        inside(o_dw, dw * e, "pairing: rearranged w_dw");
        inside(o_gpw, (size_t)n_scales * rows * 16 * e, "pairing: block-diagonal w_gpw");
    }
    return hipSuccess;
}
hipError_t launch_apply(int dt, const void* q_ms, const void* kvfrag, const float* kvscale, void* att, long n, int tpi, int n_hb,
                        float, hipStream_t) {
    const size_t states = (size_t)(n / tpi) * n_hb;
    inside(q_ms, (size_t)n * n_hb * 16 * esz(dt), "apply q_ms");
    inside(kvfrag, states * 2048, "apply operand blocks");
    inside(kvscale, states * 4, "apply scales");
    inside(att, (size_t)n * n_hb * 16 * esz(dt), "apply att");
    return hipSuccess;
}
hipError_t launch_apply_project(int dt, const void* q_ms, const void* kvfrag, const float* kvscale, const void* w_proj, void* out,
                                const void* res, long n, int tpi, int n_hb, int c_out, float, hipStream_t) {
    const size_t states = (size_t)(n / tpi) * n_hb;
    inside(q_ms, (size_t)n * n_hb * 16 * esz(dt), "apply+project q_ms");
    inside(kvfrag, states * 2048, "apply+project operand blocks");
    inside(kvscale, states * 4, "apply+project scales");
    inside(w_proj, (size_t)c_out * n_hb * 16 * esz(dt), "apply+project w_proj");
    inside(out, (size_t)n * c_out * esz(dt), "apply+project out");
    if (res) inside(res, (size_t)n * c_out * esz(dt), "apply+project residual");
    disjoint({{q_ms, (size_t)n * n_hb * 16 * esz(dt), "q_ms"}, {kvfrag, states * 2048, "operand blocks"}, {kvscale, states * 4, "scales"},
              {out, (size_t)n * c_out * esz(dt), "out"}});
    return hipSuccess;
}
hipError_t launch_transpose(int dt, const void* src, void* dst, long batch, int rows, int cols, hipStream_t) {
    inside(src, (size_t)batch * rows * cols * esz(dt), "transpose source");
    inside(dst, (size_t)batch * rows * cols * esz(dt), "transpose destination");
    return hipSuccess;
}
hipError_t launch_generic_core(int dt, const GenericArgs& a, hipStream_t) {
    const size_t e = esz(dt), T = (size_t)a.B * a.H * a.W, Ct = (size_t)a.heads * a.head_dim, S = 1 + a.n_scales;
    const size_t states = (size_t)a.B * S * a.heads, st = (size_t)a.head_dim * (a.head_dim + 1) * 4;
    inside(a.qkv, T * 3 * Ct * e, "plain core qkv");
    inside(a.q_ms, T * S * Ct * e, "plain core q_ms");
    inside(a.att, T * S * Ct * e, "plain core att");
    inside(a.partials, states * a.nchunks * st, "plain core partial states");
    inside(a.kv32, states * st, "plain core states");
    if (a.n_scales > 0) {
        size_t dw = 0;
        for (int i = 0; i < a.n_scales; ++i) dw += 3 * Ct * a.scales[i] * a.scales[i];
        inside(a.w_dw, dw * e, "plain core w_dw");
        inside(a.w_gpw, (size_t)a.n_scales * 3 * Ct * a.head_dim * e, "plain core w_gpw");
    }
    return hipSuccess;
}
hipError_t launch_ffn_dw_project(int dt, const void* h, const void* w_dw, const void* w2, const void* res, void* out, int B, int H,
                                 int W, int E, int c_out, int, hipStream_t) {
    const size_t e = esz(dt), T = (size_t)B * H * W;
    inside(h, T * E * e, "ffn expanded map");
    inside(w_dw, (size_t)E * 9 * e, "ffn w_dw");
    inside(w2, (size_t)c_out * E * e, "ffn w2");
    inside(res, T * c_out * e, "ffn residual");
    inside(out, T * c_out * e, "ffn out");
    return hipSuccess;
}
hipError_t launch_softmax_attention(int dt, const void* qkv, void* att, int B, int N, int heads, hipStream_t) {
    inside(qkv, (size_t)B * N * 3 * heads * 16 * esz(dt), "softmax qkv");
    inside(att, (size_t)B * N * heads * 16 * esz(dt), "softmax att");
    return hipSuccess;
}
hipError_t launch_linear_attention_backward(int dt, const void* qkv, const void* d_att, const float* kv32, float* partials,
                                            float* ds32, void* frag_scratch, float* scale_scratch, void* d_qkv, int B, int N,
                                            int heads, int nchunks, int, float, hipStream_t) {
    const size_t e = esz(dt), T = (size_t)B * N, st = (size_t)B * heads;
    inside(qkv, T * 3 * heads * 16 * e, "backward qkv");
    inside(d_att, T * heads * 16 * e, "backward d_att");
    inside(d_qkv, T * 3 * heads * 16 * e, "backward d_qkv");
    inside(kv32, st * 272 * 4, "backward forward states");
    inside(partials, st * nchunks * 272 * 4, "backward partial dS");
    inside(ds32, st * 272 * 4, "backward dS");
    inside(frag_scratch, st * 2048, "backward operand scratch");
    inside(scale_scratch, st * 4, "backward scale scratch");
    return hipSuccess;
}

}  // namespace msla

// ---------------------------------------------------------------- the calls
namespace {

struct Mod {
    int B, C, H, W, heads, d;
    std::vector<int> scales;
};

void expect(msla_status got, msla_status want, const char* what) {
    if (got != want) fail(std::string(what) + ": returned " + msla_error_string(got) + ", expected " + msla_error_string(want));
}

void run_module(const Mod& m, int dt) {
    const size_t e = esz(dt);
    const int ns = (int)m.scales.size(), S = 1 + ns, Ct = m.heads * m.d;
    const size_t T = (size_t)m.B * m.H * m.W;
    size_t dw = 0;
    for (int k : m.scales) dw += (size_t)3 * Ct * k * k;
    char tag[160];
    std::snprintf(tag, sizeof tag, "dt %d B %d C %d %dx%d heads %d d %d scales %d", dt, m.B, m.C, m.H, m.W, m.heads, m.d, ns);
    const int* sc = ns ? m.scales.data() : nullptr;
    const msla_dtype mdt = (msla_dtype)dt;

    size_t ws_bytes = 0;
    g_case = std::string("msla_workspace_bytes ") + tag;
    expect(msla_workspace_bytes(m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns, mdt, &ws_bytes), MSLA_OK, "workspace query");
    if (g_failures) return;

    char* x = buffer("x", T * m.C * e);
    char* w_qkv = buffer("w_qkv", (size_t)3 * Ct * m.C * e);
    char* w_dw = ns ? buffer("w_dw", dw * e) : nullptr;
    char* w_gpw = ns ? buffer("w_gpw", (size_t)ns * 3 * Ct * m.d * e) : nullptr;
    char* w_proj = buffer("w_proj", (size_t)m.C * S * Ct * e);
    char* out = buffer("out", T * m.C * e);
    char* ws = buffer("workspace", ws_bytes);

    g_case = std::string("msla_forward ") + tag;
    expect(msla_forward(x, w_qkv, w_dw, w_gpw, w_proj, out, ws, ws_bytes, m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns, 1e-15f, mdt,
                        MSLA_NHWC, nullptr), MSLA_OK, "forward");
    g_case = std::string("msla_forward, one byte of workspace short ") + tag;
    expect(msla_forward(x, w_qkv, w_dw, w_gpw, w_proj, out, ws, ws_bytes - 1, m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns, 1e-15f,
                        mdt, MSLA_NHWC, nullptr), MSLA_ERR_WORKSPACE, "forward with a short workspace");
    if (m.C <= (m.d == 32 ? 3 : 2) * Ct) {
        g_case = std::string("msla_forward NCHW ") + tag;
        expect(msla_forward(x, w_qkv, w_dw, w_gpw, w_proj, out, ws, ws_bytes, m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns, 1e-15f,
                            mdt, MSLA_NCHW, nullptr), MSLA_OK, "forward, channel-planar");
    }
    if (m.d == 16) {
        g_case = std::string("msla_forward_opts general ") + tag;
        expect(msla_forward_opts(x, w_qkv, w_dw, w_gpw, w_proj, out, ws, ws_bytes, m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns,
                                 1e-15f, mdt, MSLA_NHWC, nullptr, MSLA_OPT_GENERAL_AGGREGATION | MSLA_OPT_STATE_VALU), MSLA_OK,
               "forward, general aggregation");
        void* events[5] = {&tag, &tag, &tag, &tag, &tag};     // only handed on to the (stand-in) event call
        g_case = std::string("msla_forward_profiled ") + tag;
        expect(msla_forward_profiled(x, w_qkv, w_dw, w_gpw, w_proj, out, ws, ws_bytes, m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns,
                                     1e-15f, mdt, MSLA_NHWC, nullptr, events), MSLA_OK, "forward with stage events");
        // stage entry points on a projected map
        char* qkv = buffer("qkv", T * 3 * Ct * e);
        char* att = buffer("att", T * S * Ct * e);
        char* q_ms = buffer("q_ms out", T * S * Ct * e);
        char* kv = buffer("kv out", (size_t)m.B * S * m.heads * 272 * 4);
        g_case = std::string("msla_core_forward ") + tag;
        expect(msla_core_forward(qkv, w_dw, w_gpw, att, ws, ws_bytes, m.B, m.H, m.W, m.heads, m.d, sc, ns, 1e-15f, mdt, nullptr),
               MSLA_OK, "core forward");
        g_case = std::string("msla_multiscale_state ") + tag;
        expect(msla_multiscale_state(qkv, w_dw, w_gpw, q_ms, reinterpret_cast<float*>(kv), ws, ws_bytes, m.B, m.H, m.W, m.heads,
                                     m.d, sc, ns, mdt, nullptr), MSLA_OK, "multiscale state");
        g_case = std::string("msla_multiscale_state without q_ms ") + tag;
        expect(msla_multiscale_state(qkv, w_dw, w_gpw, nullptr, reinterpret_cast<float*>(kv), ws, ws_bytes, m.B, m.H, m.W,
                                     m.heads, m.d, sc, ns, mdt, nullptr), MSLA_OK, "multiscale state, q_ms in the workspace");
        // the whole block
        const int hidden = 4 * m.C;
        size_t bws = 0, fws = 0;
        g_case = std::string("msla_block_forward ") + tag;
        expect(msla_block_workspace_bytes(m.B, m.C, m.H, m.W, m.heads, m.d, sc, ns, hidden, mdt, &bws), MSLA_OK, "block workspace");
        expect(msla_ffn_workspace_bytes(m.B, m.C, m.H, m.W, hidden, mdt, &fws), MSLA_OK, "ffn workspace");
        char* w1 = buffer("w1", (size_t)hidden * m.C * e);
        char* wfd = buffer("w_ffn_dw", (size_t)hidden * 9 * e);
        char* w2 = buffer("w2", (size_t)m.C * hidden * e);
        char* bw = buffer("block workspace", bws);
        expect(msla_block_forward(x, w_qkv, w_dw, w_gpw, w_proj, w1, wfd, w2, out, bw, bws, m.B, m.C, m.H, m.W, m.heads, m.d, sc,
                                  ns, 1e-15f, hidden, MSLA_ACT_HSWISH, mdt, nullptr), MSLA_OK, "block forward");
        expect(msla_block_forward(x, w_qkv, w_dw, w_gpw, w_proj, w1, wfd, w2, out, bw, bws - 1, m.B, m.C, m.H, m.W, m.heads, m.d,
                                  sc, ns, 1e-15f, hidden, MSLA_ACT_HSWISH, mdt, nullptr), MSLA_ERR_WORKSPACE,
               "block forward with a short workspace");
        g_case = std::string("msla_ffn_forward ") + tag;
        char* fw = buffer("ffn workspace", fws);
        expect(msla_ffn_forward(x, w1, wfd, w2, out, fw, fws, m.B, m.C, m.H, m.W, hidden, MSLA_ACT_RELU, mdt, nullptr), MSLA_OK,
               "ffn forward");
        // backward pass and softmax on the projected map as [B, N, 3*Ct]
        size_t gws = 0;
        g_case = std::string("msla_linear_attention_backward ") + tag;
        expect(msla_linear_attention_backward_workspace_bytes(m.B, m.H * m.W, m.heads, m.d, mdt, &gws), MSLA_OK, "backward workspace");
        char* gw = buffer("backward workspace", gws);
        char* d_att = buffer("d_att", T * Ct * e);
        char* d_qkv = buffer("d_qkv", T * 3 * Ct * e);
        expect(msla_linear_attention_backward(qkv, d_att, d_qkv, gw, gws, m.B, m.H * m.W, m.heads, m.d, 1e-15f, mdt, nullptr),
               MSLA_OK, "backward");
        g_case = std::string("msla_softmax_attention ") + tag;
        expect(msla_softmax_attention(qkv, d_att, m.B, m.H * m.W, m.heads, m.d, mdt, nullptr), MSLA_OK, "softmax attention");
    }
    (void)w_proj;
    release_all();
}

}  // namespace

int main() {
    const std::vector<Mod> mods = {
        {1, 64, 32, 32, 4, 16, {5}},          // the benchmark workloads' shapes
        {1, 128, 64, 128, 8, 16, {5}},
        {1, 512, 32, 64, 32, 16, {5}},
        {1, 128, 256, 256, 8, 16, {3, 5}},
        {8, 256, 64, 128, 16, 16, {5}},
        {1, 16, 1, 1, 1, 16, {5}},            // one token
        {3, 80, 9, 20, 5, 16, {}},            // no aggregated scale, C = Ct
        {2, 48, 17, 33, 2, 16, {3, 5, 7}},    // four branches with a 7x7, C != Ct, ragged tiles
        {2, 96, 13, 21, 3, 32, {3, 7}},       // heads of 32
        {1, 128, 30, 40, 16, 8, {5}},         // heads of 8: pairs on the head-size-16 path
        {2, 64, 7, 9, 8, 8, {}},
        {5, 32, 3, 500, 2, 16, {5}},          // wide and flat
    };
    for (const Mod& m : mods)
        for (int dt = 0; dt < 3; ++dt) run_module(m, dt);
    // msla_linear on its own
    for (int dt = 0; dt < 3; ++dt) {
        const size_t e = esz(dt);
        g_case = "msla_linear";
        char* x = buffer("x", (size_t)1031 * 256 * e);
        char* w = buffer("w", (size_t)1024 * 256 * e);
        char* y = buffer("y", (size_t)1031 * 1024 * e);
        expect(msla_linear(x, w, y, 1031, 256, 1024, (msla_dtype)dt, nullptr), MSLA_OK, "linear");
        release_all();
    }
    if (g_failures) {
        std::fprintf(stderr, "%d failures\n", g_failures);
        return 1;
    }
    std::printf("dispatch driver ok: %ld extents checked\n", g_checks);
    return 0;
}
