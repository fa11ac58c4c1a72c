// Host side of the C ABI declared in include/msla.h: argument validation,
// workspace carving and the launch sequence.  No allocation, no synchronisation,
// no state that depends on a call's arguments (the only statics are per-process
// caches of device properties: the compute-unit count and "this kernel's LDS
// limit has been raised on this device"); every failure before the first
// launch leaves the stream untouched.
#include "../../include/msla.h"

#include <stdint.h>

#include "msla_kernels.h"

namespace {

constexpr int kMaxScales = 7;
constexpr unsigned kStageBits = MSLA_OPT_STAGE_PROJECT | MSLA_OPT_STAGE_AGGREGATE | MSLA_OPT_STAGE_FINALIZE |
                                MSLA_OPT_STAGE_APPLY;
// with no stage bit set every stage runs
bool stage_wanted(unsigned options, unsigned bit) { return (options & kStageBits) == 0 || (options & bit) != 0; }
constexpr size_t kAlign = 256;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

size_t elem_size(msla_dtype dt) { return dt == MSLA_F32 ? 4 : 2; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Shape {
    int B, H, W, heads, S;
    long N, T;
    int Ct;
    int n_scales;
    int scales[kMaxScales];
    // state reduction split
    int nchunks, tiles_per_chunk;
};

// Checks everything about the shape that does not involve pointers.
msla_status check_shape(int B, int H, int W, int heads, int head_dim, const int* scales, int n_scales,
                        int dt, Shape* s) {
    if (B <= 0 || H <= 0 || W <= 0 || heads <= 0 || head_dim <= 0 || n_scales < 0) return MSLA_ERR_INVALID_ARG;
    if (n_scales > 0 && scales == nullptr) return MSLA_ERR_INVALID_ARG;
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    for (int i = 0; i < n_scales; ++i)
        if (scales[i] < 1 || scales[i] % 2 == 0) return MSLA_ERR_INVALID_ARG;
    if (head_dim != 16) return MSLA_ERR_UNSUPPORTED;
    if (n_scales > kMaxScales) return MSLA_ERR_UNSUPPORTED;
    for (int i = 0; i < n_scales; ++i)
        if (scales[i] != 3 && scales[i] != 5 && scales[i] != 7) return MSLA_ERR_UNSUPPORTED;
    const long N = (long)H * W;
    const long T = N * B;
    if (N > (1L << 30) || T > (1L << 31) || (long)heads * 16 > (1L << 20)) return MSLA_ERR_UNSUPPORTED;
    s->B = B; s->H = H; s->W = W; s->heads = heads; s->S = 1 + n_scales;
    s->N = N; s->T = T; s->Ct = heads * 16; s->n_scales = n_scales;
    for (int i = 0; i < n_scales; ++i) s->scales[i] = scales[i];
    // Split each (image, head) over enough workgroups to fill the chip; every
    // workgroup then emits one partial state.  A "tile" is 8x32 (fp32) or 16x32 (16-bit types)
    // tokens for the aggregating kernels, 64 consecutive tokens when there is no aggregated scale.
    long tiles;
    long target_blocks = 1024;
    if (n_scales > 0 && dt == MSLA_F32) {
        tiles = (long)((H + msla::kAggTileH - 1) / msla::kAggTileH) * ((W + msla::kAggTileW - 1) / msla::kAggTileW);
    } else if (n_scales > 0) {
        tiles = (long)((H + msla::kAggMfmaTileH - 1) / msla::kAggMfmaTileH) *
                ((W + msla::kAggMfmaTileW - 1) / msla::kAggMfmaTileW);
        target_blocks = 256;   // one pipelined 8-wave workgroup per CU; each builds its operands once
        // (a 3x3 and a 5x5 scale share one launch: one workgroup per CU over both halves of that grid)
        if (n_scales == 2 && scales[0] + scales[1] == 8 && scales[0] != scales[1] && scales[0] != 1 && scales[1] != 1)
            target_blocks = 128;
    } else {
        tiles = (N + 63) / 64;
    }
    long want = (target_blocks + (long)B * heads - 1) / ((long)B * heads);
    if (want < 1) want = 1;
    if (want > tiles) want = tiles;
    const long tpc = (tiles + want - 1) / want;
    s->tiles_per_chunk = (int)tpc;
    s->nchunks = (int)((tiles + tpc - 1) / tpc);
    return MSLA_OK;
}

struct Workspace {
    size_t q_ms, kv_raw, partials, kv32, kvfrag, kvscale, total;
};

long kv_padded_tokens(const Shape& s) { return (s.T + 31) / 32 * 32; }

// The forward pass keeps K|V head-major ([head][token][K 16 | V 16]) when the matrix-core aggregation
// kernel will read it -- a head's tokens are then contiguous, which that kernel's loads like (-2 us
// on the headline workload) -- and the map fits 32-bit byte offsets; token-major otherwise.
bool kv_head_major(const Shape& s, msla_dtype dt) {
    return dt != MSLA_F32 && s.n_scales > 0 && (size_t)kv_padded_tokens(s) * 2 * s.Ct * elem_size(dt) < (1ull << 31);
}

// with_maps = false: only the small per-state buffers (for an entry point whose caller supplies the
// token maps itself)
Workspace carve(const Shape& s, msla_dtype dt, bool with_maps = true) {
    const size_t e = elem_size(dt);
    const size_t n_states = (size_t)s.B * s.S * s.heads;
    Workspace w;
    size_t off = 0;
    w.q_ms = off;     off += with_maps ? align_up((size_t)s.T * s.S * s.Ct * e) : 0;
    // (token count rounded up to whole projection tiles: the head-major form of this map pads each head)
    w.kv_raw = off;   off += with_maps ? align_up((size_t)kv_padded_tokens(s) * 2 * s.Ct * e) : 0;
    w.partials = off; off += align_up(n_states * s.nchunks * 272 * sizeof(float));
    w.kv32 = off;     off += align_up(n_states * 272 * sizeof(float));
    w.kvfrag = off;   off += align_up(n_states * 2048);
    w.kvscale = off;  off += align_up(n_states * sizeof(float));
    w.total = off;
    return w;
}

size_t dw_weight_elems(const Shape& s, int upto) {
    size_t n = 0;
    for (int i = 0; i < upto; ++i) n += (size_t)3 * s.Ct * s.scales[i] * s.scales[i];
    return n;
}

// Aggregation + state for all branches.  The raw maps are given as three strided views.
msla_status run_state(const Shape& s, msla_dtype dt, const void* q, long q_ts, int q_hs, const void* k,
                      long k_ts, int k_hs, const void* v, long v_ts, int v_hs, const void* w_dw,
                      const void* w_gpw, char* ws, const Workspace& wo, void* q_ms, int copy_raw_q,
                      hipStream_t stream, unsigned options = 0, void* event_before_finalize = nullptr,
                      int state_split = 0) {
    const size_t e = elem_size(dt);
    msla::AggregateArgs a;
    a.q = q; a.k = k; a.v = v;
    a.q_ts = q_ts; a.k_ts = k_ts; a.v_ts = v_ts;
    a.q_hs = q_hs; a.k_hs = k_hs; a.v_hs = v_hs;
    a.q_ms = q_ms;
    a.partials = reinterpret_cast<float*>(ws + wo.partials);
    a.B = s.B; a.H = s.H; a.W = s.W; a.heads = s.heads; a.S = s.S;
    a.nchunks = s.nchunks; a.tiles_per_chunk = s.tiles_per_chunk;
    const bool aggregate = stage_wanted(options, MSLA_OPT_STAGE_AGGREGATE);
    if (s.n_scales == 0 && aggregate) {
        a.w_dw = nullptr; a.w_gpw = nullptr; a.ks = 0; a.branch = 0; a.do_raw = 1; a.copy_raw_q = copy_raw_q;
        a.state_valu = (options & MSLA_OPT_STATE_VALU) ? 1 : 0;
        if (msla::launch_raw_state((int)dt, a, stream) != hipSuccess) return MSLA_ERR_LAUNCH;
    }
    auto aim = [&](msla::AggregateArgs& g, int i) {
        g.w_dw = static_cast<const char*>(w_dw) + dw_weight_elems(s, i) * e;
        g.w_gpw = static_cast<const char*>(w_gpw) + (size_t)i * 3 * s.Ct * 16 * e;
        g.ks = s.scales[i];
        g.branch = i + 1;
        g.do_raw = (i == 0);
        g.copy_raw_q = (i == 0) ? copy_raw_q : 0;
    };
    int first = 0;
    if (aggregate && s.n_scales == 2 && dt != MSLA_F32 && !(options & MSLA_OPT_GENERAL_AGGREGATION)) {
        // a 3x3 and a 5x5 scale: both in one launch, so the compute units do not drain between them
        msla::AggregateArgs a0 = a, a1 = a;
        aim(a0, 0);
        aim(a1, 1);
        const hipError_t e_pair = msla::launch_aggregate_mfma_pair((int)dt, a0, a1, stream);
        if (e_pair == hipSuccess) first = 2;
        else if (e_pair != hipErrorNotSupported) return MSLA_ERR_LAUNCH;
    }
    for (int i = first; i < s.n_scales && aggregate; ++i) {
        a.w_dw = static_cast<const char*>(w_dw) + dw_weight_elems(s, i) * e;
        a.w_gpw = static_cast<const char*>(w_gpw) + (size_t)i * 3 * s.Ct * 16 * e;
        a.ks = s.scales[i];
        a.branch = i + 1;
        a.do_raw = (i == 0);
        a.copy_raw_q = (i == 0) ? copy_raw_q : 0;
        // (MSLA_OPT_GENERAL_AGGREGATION sends every case to the general kernel: that is how the tests
        // reach the path below without a 2 GiB image)
        const bool general = dt == MSLA_F32 || (options & MSLA_OPT_GENERAL_AGGREGATION);
        hipError_t e_launch = (dt == MSLA_F32) ? msla::launch_aggregate((int)dt, a, stream)
                              : general        ? hipErrorNotSupported
                                               : msla::launch_aggregate_mfma((int)dt, a, stream);
        // an image whose maps exceed the matrix-core kernel's 32-bit offsets takes the general kernel,
        // whose tiles are half as high: the same number of chunks, twice the tiles in each
        if (e_launch == hipErrorNotSupported) {
            msla::AggregateArgs g = a;
            const long tiles = (long)((s.H + msla::kAggTileH - 1) / msla::kAggTileH) *
                               ((s.W + msla::kAggTileW - 1) / msla::kAggTileW);
            g.tiles_per_chunk = (int)((tiles + a.nchunks - 1) / a.nchunks);
            e_launch = msla::launch_aggregate((int)dt, g, stream);
        }
        if (e_launch != hipSuccess) return MSLA_ERR_LAUNCH;
    }
    if (event_before_finalize &&
        hipEventRecord(static_cast<hipEvent_t>(event_before_finalize), stream) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    const int n_states = s.B * s.S * s.heads;
    if (stage_wanted(options, MSLA_OPT_STAGE_FINALIZE) &&
        msla::launch_state_finalize((int)dt, a.partials, reinterpret_cast<float*>(ws + wo.kv32), ws + wo.kvfrag,
                                    reinterpret_cast<float*>(ws + wo.kvscale), n_states, s.nchunks,
                                    stream, state_split) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

}  // namespace

namespace msla {
int compute_units() {
    static int cached = 0;      // a device property, not call state; benign if two threads race to set it
    if (cached <= 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;            // MI355X
        cached = n;
    }
    return cached;
}
}  // namespace msla

namespace {

// ---- head sizes 8 and 32: projection -> generic core (k_generic.hip) -> projection
struct GenericPlan {
    long T;
    int Ct, S, nchunks;
    size_t qkv, q_ms, att, partials, kv32, total;
};

bool generic_head_dim(int head_dim) { return head_dim == 8 || head_dim == 32; }

msla_status generic_plan(int B, int C, int H, int W, int heads, int head_dim, const int* scales, int n_scales, int dt,
                         GenericPlan* p) {
    if (B <= 0 || C <= 0 || H <= 0 || W <= 0 || heads <= 0 || n_scales < 0) return MSLA_ERR_INVALID_ARG;
    if (n_scales > 0 && scales == nullptr) return MSLA_ERR_INVALID_ARG;
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    for (int i = 0; i < n_scales; ++i)
        if (scales[i] < 1 || scales[i] % 2 == 0) return MSLA_ERR_INVALID_ARG;
    if (n_scales > kMaxScales) return MSLA_ERR_UNSUPPORTED;
    for (int i = 0; i < n_scales; ++i)
        if (scales[i] != 3 && scales[i] != 5 && scales[i] != 7) return MSLA_ERR_UNSUPPORTED;
    const long N = (long)H * W;
    if (N > (1L << 30) || N * B > (1L << 31) || (long)heads * head_dim > (1L << 20)) return MSLA_ERR_UNSUPPORTED;
    if (C % 16 != 0 || (heads * head_dim) % 16 != 0) return MSLA_ERR_UNSUPPORTED;
    const size_t e = elem_size((msla_dtype)dt);
    p->T = N * B; p->Ct = heads * head_dim; p->S = 1 + n_scales;
    const long groups = (N + 63) / 64;
    long want = (512 + (long)B * heads - 1) / ((long)B * heads);
    if (want > groups) want = groups;
    if (want < 1) want = 1;
    p->nchunks = (int)want;
    const size_t n_states = (size_t)B * p->S * heads, state = (size_t)head_dim * (head_dim + 1) * sizeof(float);
    size_t off = 0;
    p->qkv = off;      off += align_up((size_t)p->T * 3 * p->Ct * e);
    p->q_ms = off;     off += align_up((size_t)p->T * p->S * p->Ct * e);
    p->att = off;      off += align_up((size_t)p->T * p->S * p->Ct * e);
    p->partials = off; off += align_up(n_states * p->nchunks * state);
    p->kv32 = off;     off += align_up(n_states * state);
    p->total = off;
    return MSLA_OK;
}

// Head size 8 with an even number of heads runs on the head-size-16 kernels, two heads to one of 16
// (launch_pair_head8_weights, launch_state_finalize with split = 8).  Its workspace: the three rearranged
// weight arrays, then the workspace of the head-size-16 module.
struct Paired8Plan {
    size_t w_qkv, w_dw, w_gpw, inner, inner_bytes, total;
};
bool paired8(int heads, int head_dim) { return head_dim == 8 && heads > 0 && heads % 2 == 0; }
msla_status paired8_plan(int B, int C, int H, int W, int heads, const int* scales, int n_scales, msla_dtype dt, Paired8Plan* p) {
    Shape s;
    const msla_status st = check_shape(B, H, W, heads / 2, 16, scales, n_scales, (int)dt, &s);
    if (st != MSLA_OK) return st;
    if (C <= 0 || C % 16 != 0) return MSLA_ERR_UNSUPPORTED;
    const size_t e = elem_size(dt);
    size_t off = 0;
    p->w_qkv = off; off += align_up((size_t)3 * s.Ct * C * e);
    p->w_dw = off;  off += align_up(dw_weight_elems(s, n_scales) * e + 16);
    p->w_gpw = off; off += align_up((size_t)n_scales * 3 * s.Ct * 16 * e + 16);
    p->inner = off;
    p->inner_bytes = carve(s, dt).total;
    p->total = off + p->inner_bytes;
    return MSLA_OK;
}

msla_status generic_forward(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw, const void* w_proj,
                            void* out, void* workspace, size_t workspace_bytes, int B, int C, int H, int W, int heads,
                            int head_dim, const int* scales, int n_scales, float eps, msla_dtype dt, msla_layout layout,
                            hipStream_t hs) {
    GenericPlan p;
    const msla_status st = generic_plan(B, C, H, W, heads, head_dim, scales, n_scales, (int)dt, &p);
    if (st != MSLA_OK) return st;
    if (workspace_bytes < p.total) return MSLA_ERR_WORKSPACE;
    // channel-planar x / out: x is turned into token-major form in `out` (free until the last kernel), the
    // token-major result is parked where the projected Q/K/V lived and turned back into `out`
    if (layout == MSLA_NCHW && C > 3 * p.Ct) return MSLA_ERR_UNSUPPORTED;
    char* ws = static_cast<char*>(workspace);
    void* out_tok = out;
    if (layout == MSLA_NCHW) {
        if (msla::launch_transpose((int)dt, x, out, B, C, H * W, hs) != hipSuccess) return MSLA_ERR_LAUNCH;
        x = out;
        out_tok = ws + p.qkv;
    }
    if (msla::launch_linear((int)dt, x, w_qkv, ws + p.qkv, p.T, C, 3 * p.Ct, hs) != hipSuccess) return MSLA_ERR_LAUNCH;
    msla::GenericArgs a;
    a.qkv = ws + p.qkv; a.w_dw = w_dw; a.w_gpw = w_gpw; a.q_ms = ws + p.q_ms;
    a.partials = reinterpret_cast<float*>(ws + p.partials); a.kv32 = reinterpret_cast<float*>(ws + p.kv32);
    a.att = ws + p.att;
    a.B = B; a.H = H; a.W = W; a.heads = heads; a.head_dim = head_dim; a.n_scales = n_scales;
    for (int i = 0; i < n_scales; ++i) a.scales[i] = scales[i];
    a.nchunks = p.nchunks; a.eps = eps;
    if (msla::launch_generic_core((int)dt, a, hs) != hipSuccess) return MSLA_ERR_LAUNCH;
    if (msla::launch_linear((int)dt, ws + p.att, w_proj, out_tok, p.T, p.S * p.Ct, C, hs) != hipSuccess) return MSLA_ERR_LAUNCH;
    if (layout == MSLA_NCHW && msla::launch_transpose((int)dt, out_tok, out, B, H * W, C, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

}  // namespace

namespace msla {
int multiscale_state_small(const void* qkv, const void* w_dw, const void* w_gpw, void* q_ms, float* kv,
                           void* scratch, size_t scratch_bytes, int B, int H, int W, int heads, int head_dim,
                           const int* scales, int n_scales, int dt, hipStream_t stream);
}

extern "C" {

const char* msla_error_string(msla_status status) {
    switch (status) {
        case MSLA_OK: return "MSLA_OK";
        case MSLA_ERR_INVALID_ARG: return "MSLA_ERR_INVALID_ARG: null/misaligned pointer, non-positive size, even kernel size, negative eps or unknown enum";
        case MSLA_ERR_UNSUPPORTED: return "MSLA_ERR_UNSUPPORTED: shape, head size, kernel size or layout not covered by the kernels";
        case MSLA_ERR_WORKSPACE: return "MSLA_ERR_WORKSPACE: workspace smaller than msla_workspace_bytes reports";
        case MSLA_ERR_LAUNCH: return "MSLA_ERR_LAUNCH: HIP error while enqueueing";
    }
    return "unknown msla_status";
}

msla_status msla_workspace_bytes(int B, int C, int H, int W, int heads, int head_dim, const int* scales,
                                 int n_scales, msla_dtype dt, size_t* bytes) {
    if (bytes == nullptr || C <= 0) return MSLA_ERR_INVALID_ARG;
    if (generic_head_dim(head_dim)) {
        GenericPlan p;
        const msla_status gst = generic_plan(B, C, H, W, heads, head_dim, scales, n_scales, (int)dt, &p);
        if (gst != MSLA_OK) return gst;
        if (paired8(heads, head_dim)) {
            Paired8Plan pp;
            const msla_status pst = paired8_plan(B, C, H, W, heads, scales, n_scales, dt, &pp);
            if (pst != MSLA_OK) return pst;
            *bytes = pp.total;
            return MSLA_OK;
        }
        *bytes = p.total;
        return MSLA_OK;
    }
    Shape s;
    const msla_status st = check_shape(B, H, W, heads, head_dim, scales, n_scales, (int)dt, &s);
    if (st != MSLA_OK) return st;
    if (C % 16 != 0) return MSLA_ERR_UNSUPPORTED;
    *bytes = carve(s, dt).total;
    return MSLA_OK;
}

static msla_status forward_impl(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw,
                                const void* w_proj, void* out, void* workspace, size_t workspace_bytes, int B,
                                int C, int H, int W, int heads, int head_dim, const int* scales, int n_scales,
                                float eps, msla_dtype dt, msla_layout layout, void* stream,
                                void* const* events, unsigned options, const void* residual = nullptr,
                                int state_split = 0) {
    if (!x || !w_qkv || !w_proj || !out || !workspace || C <= 0) return MSLA_ERR_INVALID_ARG;
    if (options & ~(MSLA_OPT_GENERAL_AGGREGATION | MSLA_OPT_STATE_VALU | kStageBits)) return MSLA_ERR_INVALID_ARG;
    if ((options & kStageBits) && layout != MSLA_NHWC) return MSLA_ERR_UNSUPPORTED;
    if (n_scales > 0 && (!w_dw || !w_gpw)) return MSLA_ERR_INVALID_ARG;
    if (!(eps >= 0.0f)) return MSLA_ERR_INVALID_ARG;
    if (layout != MSLA_NHWC && layout != MSLA_NCHW) return MSLA_ERR_INVALID_ARG;
    if (generic_head_dim(head_dim)) {
        // head sizes 8 and 32: no options, no stage events, no residual
        if (!aligned16(x) || !aligned16(w_qkv) || !aligned16(w_proj) || !aligned16(out) || !aligned16(workspace) ||
            !aligned16(w_dw) || !aligned16(w_gpw))
            return MSLA_ERR_INVALID_ARG;
        if (options != 0 || events != nullptr || residual != nullptr) return MSLA_ERR_UNSUPPORTED;
        if (layout != MSLA_NHWC && !paired8(heads, head_dim) && head_dim != 32) return MSLA_ERR_UNSUPPORTED;
        if (paired8(heads, head_dim)) {
            // two heads of 8 as one head of 16: rearranged weights, then the head-size-16 module
            GenericPlan gp;     // (argument checks shared with the plain path)
            msla_status pst = generic_plan(B, C, H, W, heads, head_dim, scales, n_scales, (int)dt, &gp);
            if (pst != MSLA_OK) return pst;
            Paired8Plan pp;
            pst = paired8_plan(B, C, H, W, heads, scales, n_scales, dt, &pp);
            if (pst != MSLA_OK) return pst;
            if (workspace_bytes < pp.total) return MSLA_ERR_WORKSPACE;
            char* pws = static_cast<char*>(workspace);
            if (msla::launch_pair_head8_weights((int)dt, w_qkv, w_dw, w_gpw, pws + pp.w_qkv, pws + pp.w_dw, pws + pp.w_gpw, C,
                                                heads, scales, n_scales, static_cast<hipStream_t>(stream)) != hipSuccess)
                return MSLA_ERR_LAUNCH;
            return forward_impl(x, pws + pp.w_qkv, n_scales > 0 ? pws + pp.w_dw : nullptr,
                                n_scales > 0 ? pws + pp.w_gpw : nullptr, w_proj, out, pws + pp.inner, pp.inner_bytes, B, C, H, W,
                                heads / 2, 16, scales, n_scales, eps, dt, layout, stream, nullptr, 0u, nullptr, 8);
        }
        return generic_forward(x, w_qkv, w_dw, w_gpw, w_proj, out, workspace, workspace_bytes, B, C, H, W, heads, head_dim,
                               scales, n_scales, eps, dt, layout, static_cast<hipStream_t>(stream));
    }
    if (!aligned16(x) || !aligned16(w_qkv) || !aligned16(w_proj) || !aligned16(out) || !aligned16(workspace) ||
        !aligned16(w_dw) || !aligned16(w_gpw))
        return MSLA_ERR_INVALID_ARG;
    Shape s;
    msla_status st = check_shape(B, H, W, heads, head_dim, scales, n_scales, (int)dt, &s);
    if (st != MSLA_OK) return st;
    if (C % 16 != 0) return MSLA_ERR_UNSUPPORTED;
    // channel-planar x / out: the result is parked where K|V lived, which must be large enough
    if (layout == MSLA_NCHW && C > 2 * s.Ct) return MSLA_ERR_UNSUPPORTED;
    const Workspace wo = carve(s, dt);
    if (workspace_bytes < wo.total) return MSLA_ERR_WORKSPACE;

    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const size_t e = elem_size(dt);
    void* q_ms = ws + wo.q_ms;
    char* kv_raw = ws + wo.kv_raw;
    const long q_ms_ts = (long)s.S * s.Ct;

    auto mark = [&](int i) -> bool {
        return events == nullptr || hipEventRecord(static_cast<hipEvent_t>(events[i]), hs) == hipSuccess;
    };
    if (!mark(0)) return MSLA_ERR_LAUNCH;
    // The kernels work token-major.  A channel-planar x is first turned into token-major form in
    // `out` (free until the last kernel); the token-major result is then parked in the K|V area
    // (dead after the aggregation pass) and turned back into `out`.
    const void* x_tok = x;
    void* out_tok = out;
    if (layout == MSLA_NCHW) {
        if (msla::launch_transpose((int)dt, x, out, s.B, C, (int)s.N, hs) != hipSuccess) return MSLA_ERR_LAUNCH;
        x_tok = out;
        out_tok = kv_raw;
    }
    // Q/K/V projection; raw Q lands in the branch-0 columns of the multi-scale Q map
    const bool hm = kv_head_major(s, dt);
    const long kv_ts = hm ? 32 : 2L * s.Ct;                       // elements from token to token
    const long kv_hs = hm ? kv_padded_tokens(s) * 32 : 32;        // ... from head to head
    const long kv_span = hm ? kv_padded_tokens(s) * 2 * s.Ct : s.T * 2 * s.Ct;
    if (stage_wanted(options, MSLA_OPT_STAGE_PROJECT) &&
        msla::launch_qkv_project((int)dt, x_tok, w_qkv, q_ms, q_ms_ts, kv_raw, kv_ts, kv_hs, kv_span, s.T, C, s.heads,
                                 hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    if (!mark(1)) return MSLA_ERR_LAUNCH;
    // aggregation + Eq. (3) state
    st = run_state(s, dt, q_ms, q_ms_ts, 16, kv_raw, kv_ts, (int)kv_hs, kv_raw + 16 * e, kv_ts, (int)kv_hs, w_dw, w_gpw,
                   ws, wo, q_ms, /*copy_raw_q=*/0, hs, options, events ? events[2] : nullptr, state_split);
    if (st != MSLA_OK) return st;
    if (!mark(3)) return MSLA_ERR_LAUNCH;
    // normalise-and-apply fused with the output projection
    if (stage_wanted(options, MSLA_OPT_STAGE_APPLY) &&
        msla::launch_apply_project((int)dt, q_ms, ws + wo.kvfrag, reinterpret_cast<float*>(ws + wo.kvscale),
                                   w_proj, out_tok, residual, s.T, (int)s.N, s.S * s.heads, C, eps, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    if (layout == MSLA_NCHW &&
        msla::launch_transpose((int)dt, out_tok, out, s.B, (int)s.N, C, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    if (!mark(4)) return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

msla_status msla_forward(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw,
                         const void* w_proj, void* out, void* workspace, size_t workspace_bytes, int B, int C,
                         int H, int W, int heads, int head_dim, const int* scales, int n_scales, float eps,
                         msla_dtype dt, msla_layout layout, void* stream) {
    return forward_impl(x, w_qkv, w_dw, w_gpw, w_proj, out, workspace, workspace_bytes, B, C, H, W, heads,
                        head_dim, scales, n_scales, eps, dt, layout, stream, nullptr, 0u);
}

msla_status msla_forward_opts(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw,
                              const void* w_proj, void* out, void* workspace, size_t workspace_bytes, int B, int C,
                              int H, int W, int heads, int head_dim, const int* scales, int n_scales, float eps,
                              msla_dtype dt, msla_layout layout, void* stream, unsigned options) {
    return forward_impl(x, w_qkv, w_dw, w_gpw, w_proj, out, workspace, workspace_bytes, B, C, H, W, heads,
                        head_dim, scales, n_scales, eps, dt, layout, stream, nullptr, options);
}

msla_status msla_forward_profiled(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw,
                                  const void* w_proj, void* out, void* workspace, size_t workspace_bytes, int B,
                                  int C, int H, int W, int heads, int head_dim, const int* scales, int n_scales,
                                  float eps, msla_dtype dt, msla_layout layout, void* stream,
                                  void* const* events) {
    if (events == nullptr) return MSLA_ERR_INVALID_ARG;
    for (int i = 0; i < 5; ++i)
        if (events[i] == nullptr) return MSLA_ERR_INVALID_ARG;
    return forward_impl(x, w_qkv, w_dw, w_gpw, w_proj, out, workspace, workspace_bytes, B, C, H, W, heads,
                        head_dim, scales, n_scales, eps, dt, layout, stream, events, 0u);
}

// Shared by msla_multiscale_state and its allocation-free variant: `small` says that `workspace`
// holds only the per-state buffers (then q_ms_out must be given).
static msla_status multiscale_state_impl(const void* qkv, const void* w_dw, const void* w_gpw, void* q_ms_out,
                                         float* kv, void* workspace, size_t workspace_bytes, int B, int H, int W,
                                         int heads, int head_dim, const int* scales, int n_scales, msla_dtype dt,
                                         void* stream, bool small) {
    if (!qkv || !workspace || !kv || (small && !q_ms_out)) return MSLA_ERR_INVALID_ARG;
    if (n_scales > 0 && (!w_dw || !w_gpw)) return MSLA_ERR_INVALID_ARG;
    if (!aligned16(qkv) || !aligned16(workspace) || !aligned16(w_dw) || !aligned16(w_gpw) ||
        !aligned16(q_ms_out) || !aligned16(kv))
        return MSLA_ERR_INVALID_ARG;
    Shape s;
    msla_status st = check_shape(B, H, W, heads, head_dim, scales, n_scales, (int)dt, &s);
    if (st != MSLA_OK) return st;
    const Workspace wo = carve(s, dt, !small);
    if (workspace_bytes < wo.total) return MSLA_ERR_WORKSPACE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const size_t e = elem_size(dt);
    const char* base = static_cast<const char*>(qkv);
    void* q_ms = q_ms_out ? q_ms_out : static_cast<void*>(ws + wo.q_ms);
    st = run_state(s, dt, base, 3L * s.Ct, 48, base + 16 * e, 3L * s.Ct, 48, base + 32 * e, 3L * s.Ct, 48, w_dw,
                   w_gpw, ws, wo, q_ms, /*copy_raw_q=*/1, hs);
    if (st != MSLA_OK) return st;
    const size_t n_states = (size_t)s.B * s.S * s.heads;
    if (hipMemcpyAsync(kv, ws + wo.kv32, n_states * 272 * sizeof(float), hipMemcpyDeviceToDevice, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

msla_status msla_multiscale_state(const void* qkv, const void* w_dw, const void* w_gpw, void* q_ms_out,
                                  float* kv, void* workspace, size_t workspace_bytes, int B, int H, int W,
                                  int heads, int head_dim, const int* scales, int n_scales, msla_dtype dt,
                                  void* stream) {
    return multiscale_state_impl(qkv, w_dw, w_gpw, q_ms_out, kv, workspace, workspace_bytes, B, H, W, heads,
                                 head_dim, scales, n_scales, dt, stream, /*small=*/false);
}

msla_status msla_core_forward(const void* qkv, const void* w_dw, const void* w_gpw, void* att, void* workspace,
                              size_t workspace_bytes, int B, int H, int W, int heads, int head_dim,
                              const int* scales, int n_scales, float eps, msla_dtype dt, void* stream) {
    if (!qkv || !att || !workspace) return MSLA_ERR_INVALID_ARG;
    if (n_scales > 0 && (!w_dw || !w_gpw)) return MSLA_ERR_INVALID_ARG;
    if (!(eps >= 0.0f)) return MSLA_ERR_INVALID_ARG;
    if (!aligned16(qkv) || !aligned16(att) || !aligned16(workspace) || !aligned16(w_dw) || !aligned16(w_gpw))
        return MSLA_ERR_INVALID_ARG;
    Shape s;
    msla_status st = check_shape(B, H, W, heads, head_dim, scales, n_scales, (int)dt, &s);
    if (st != MSLA_OK) return st;
    const Workspace wo = carve(s, dt);
    if (workspace_bytes < wo.total) return MSLA_ERR_WORKSPACE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    const size_t e = elem_size(dt);
    const char* base = static_cast<const char*>(qkv);
    void* q_ms = ws + wo.q_ms;
    st = run_state(s, dt, base, 3L * s.Ct, 48, base + 16 * e, 3L * s.Ct, 48, base + 32 * e, 3L * s.Ct, 48, w_dw,
                   w_gpw, ws, wo, q_ms, /*copy_raw_q=*/1, hs);
    if (st != MSLA_OK) return st;
    if (msla::launch_apply((int)dt, q_ms, ws + wo.kvfrag, reinterpret_cast<float*>(ws + wo.kvscale), att, s.T,
                           (int)s.N, s.S * s.heads, eps, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

// ---- FFN+DWConv and the whole building block
static bool ffn_shape_ok(int B, int C, int H, int W, int hidden) {
    return B > 0 && C > 0 && H > 0 && W > 0 && hidden > 0;
}
static size_t ffn_ws_bytes(long T, int hidden, msla_dtype dt) { return align_up((size_t)T * hidden * elem_size(dt)); }

msla_status msla_ffn_workspace_bytes(int B, int C, int H, int W, int hidden, msla_dtype dt, size_t* bytes) {
    if (!bytes || !ffn_shape_ok(B, C, H, W, hidden)) return MSLA_ERR_INVALID_ARG;
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    if (C % 16 != 0 || hidden % 16 != 0 || (long)B * H * W > (1L << 31)) return MSLA_ERR_UNSUPPORTED;
    *bytes = ffn_ws_bytes((long)B * H * W, hidden, dt);
    return MSLA_OK;
}

msla_status msla_ffn_forward(const void* y, const void* w1, const void* w_dw, const void* w2, void* out,
                             void* workspace, size_t workspace_bytes, int B, int C, int H, int W, int hidden,
                             msla_act act, msla_dtype dt, void* stream) {
    if (!y || !w1 || !w_dw || !w2 || !out || !workspace || !ffn_shape_ok(B, C, H, W, hidden)) return MSLA_ERR_INVALID_ARG;
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    if (act != MSLA_ACT_RELU && act != MSLA_ACT_HSWISH) return MSLA_ERR_INVALID_ARG;
    if (!aligned16(y) || !aligned16(w1) || !aligned16(w_dw) || !aligned16(w2) || !aligned16(out) || !aligned16(workspace))
        return MSLA_ERR_INVALID_ARG;
    const long T = (long)B * H * W;
    if (C % 16 != 0 || hidden % 16 != 0 || T > (1L << 31)) return MSLA_ERR_UNSUPPORTED;
    if (workspace_bytes < ffn_ws_bytes(T, hidden, dt)) return MSLA_ERR_WORKSPACE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* h_pre = static_cast<char*>(workspace);
    if (msla::launch_linear_act((int)dt, y, w1, h_pre, T, C, hidden, (int)act, hs) != hipSuccess) return MSLA_ERR_LAUNCH;
    // depthwise 3x3 + activation + hidden -> C projection + residual in one kernel (the depthwise result stays on chip)
    if (msla::launch_ffn_dw_project((int)dt, h_pre, w_dw, w2, y, out, B, H, W, hidden, C, (int)act, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

msla_status msla_block_workspace_bytes(int B, int C, int H, int W, int heads, int head_dim, const int* scales,
                                       int n_scales, int hidden, msla_dtype dt, size_t* bytes) {
    size_t a = 0, f = 0;
    msla_status st = msla_workspace_bytes(B, C, H, W, heads, head_dim, scales, n_scales, dt, &a);
    if (st != MSLA_OK) return st;
    st = msla_ffn_workspace_bytes(B, C, H, W, hidden, dt, &f);
    if (st != MSLA_OK) return st;
    if (!bytes) return MSLA_ERR_INVALID_ARG;
    // the attention module's workspace is dead once y = x + MSLA(x) exists, so the FFN reuses it
    *bytes = align_up((size_t)B * H * W * C * elem_size(dt)) + (a > f ? a : f);
    return MSLA_OK;
}

msla_status msla_block_forward(const void* x, const void* w_qkv, const void* w_dw, const void* w_gpw,
                               const void* w_proj, const void* w1, const void* w_ffn_dw, const void* w2, void* out,
                               void* workspace, size_t workspace_bytes, int B, int C, int H, int W, int heads,
                               int head_dim, const int* scales, int n_scales, float eps, int hidden, msla_act act,
                               msla_dtype dt, void* stream) {
    size_t need = 0;
    const msla_status sz = msla_block_workspace_bytes(B, C, H, W, heads, head_dim, scales, n_scales, hidden, dt, &need);
    if (sz != MSLA_OK) return sz;
    if (!workspace || !x || !out || !w1 || !w_ffn_dw || !w2 || !aligned16(workspace)) return MSLA_ERR_INVALID_ARG;
    if (act != MSLA_ACT_RELU && act != MSLA_ACT_HSWISH) return MSLA_ERR_INVALID_ARG;
    if (workspace_bytes < need) return MSLA_ERR_WORKSPACE;
    const size_t y_bytes = align_up((size_t)B * H * W * C * elem_size(dt));
    char* ybuf = static_cast<char*>(workspace);
    char* rest = ybuf + y_bytes;
    // y = x + MSLA(x) in one rounding: x joins the output projection's fp32 sums as a residual
    const msla_status st = forward_impl(x, w_qkv, w_dw, w_gpw, w_proj, ybuf, rest, workspace_bytes - y_bytes, B, C, H, W,
                                        heads, head_dim, scales, n_scales, eps, dt, MSLA_NHWC, stream, nullptr, 0u, x);
    if (st != MSLA_OK) return st;
    return msla_ffn_forward(ybuf, w1, w_ffn_dw, w2, out, rest, workspace_bytes - y_bytes, B, C, H, W, hidden, act, dt, stream);
}

msla_status msla_linear_attention_backward_workspace_bytes(int B, int N, int heads, int head_dim, msla_dtype dt,
                                                           size_t* bytes) {
    if (!bytes) return MSLA_ERR_INVALID_ARG;
    Shape s;
    const msla_status st = check_shape(B, 1, N, heads, head_dim, nullptr, 0, (int)dt, &s);
    if (st != MSLA_OK) return st;
    *bytes = 2 * carve(s, dt, /*with_maps=*/false).total;
    return MSLA_OK;
}

msla_status msla_linear_attention_backward(const void* qkv, const void* d_att, void* d_qkv, void* workspace,
                                           size_t workspace_bytes, int B, int N, int heads, int head_dim, float eps,
                                           msla_dtype dt, void* stream) {
    if (!qkv || !d_att || !d_qkv || !workspace) return MSLA_ERR_INVALID_ARG;
    if (!(eps >= 0.0f)) return MSLA_ERR_INVALID_ARG;
    if (!aligned16(qkv) || !aligned16(d_att) || !aligned16(d_qkv) || !aligned16(workspace)) return MSLA_ERR_INVALID_ARG;
    Shape s;
    msla_status st = check_shape(B, 1, N, heads, head_dim, nullptr, 0, (int)dt, &s);
    if (st != MSLA_OK) return st;
    const Workspace wo = carve(s, dt, /*with_maps=*/false);
    if (workspace_bytes < 2 * wo.total) return MSLA_ERR_WORKSPACE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    char* ws2 = ws + wo.total;
    const size_t e = elem_size(dt);
    const char* base = static_cast<const char*>(qkv);
    // forward state S of Eq. (3) (the library's own state kernels), then dS, then the three gradients
    st = run_state(s, dt, base, 3L * s.Ct, 48, base + 16 * e, 3L * s.Ct, 48, base + 32 * e, 3L * s.Ct, 48, nullptr, nullptr,
                   ws, wo, nullptr, /*copy_raw_q=*/0, hs);
    if (st != MSLA_OK) return st;
    if (msla::launch_linear_attention_backward((int)dt, qkv, d_att, reinterpret_cast<const float*>(ws + wo.kv32),
                                               reinterpret_cast<float*>(ws2 + wo.partials),
                                               reinterpret_cast<float*>(ws2 + wo.kv32), ws2 + wo.kvfrag,
                                               reinterpret_cast<float*>(ws2 + wo.kvscale), d_qkv, B, N, heads, s.nchunks,
                                               s.tiles_per_chunk, eps, hs) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

msla_status msla_softmax_attention(const void* qkv, void* att, int B, int N, int heads, int head_dim, msla_dtype dt,
                                   void* stream) {
    if (!qkv || !att || B <= 0 || N <= 0 || heads <= 0 || head_dim <= 0) return MSLA_ERR_INVALID_ARG;
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    if (!aligned16(qkv) || !aligned16(att)) return MSLA_ERR_INVALID_ARG;
    if (head_dim != 16 || (long)B * N > (1L << 31) || (long)heads * 16 > (1L << 20)) return MSLA_ERR_UNSUPPORTED;
    if (msla::launch_softmax_attention((int)dt, qkv, att, B, N, heads, static_cast<hipStream_t>(stream)) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

msla_status msla_linear(const void* x, const void* w, void* y, long n_tokens, int c_in, int c_out,
                        msla_dtype dt, void* stream) {
    if (!x || !w || !y || n_tokens <= 0 || c_in <= 0 || c_out <= 0) return MSLA_ERR_INVALID_ARG;
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return MSLA_ERR_INVALID_ARG;
    if (c_in % 16 != 0 || c_out % 16 != 0 || n_tokens > (1L << 31)) return MSLA_ERR_UNSUPPORTED;
    if (msla::launch_linear((int)dt, x, w, y, n_tokens, c_in, c_out, static_cast<hipStream_t>(stream)) != hipSuccess)
        return MSLA_ERR_LAUNCH;
    return MSLA_OK;
}

}  // extern "C"

int msla::multiscale_state_small(const void* qkv, const void* w_dw, const void* w_gpw, void* q_ms, float* kv,
                                 void* scratch, size_t scratch_bytes, int B, int H, int W, int heads,
                                 int head_dim, const int* scales, int n_scales, int dt, hipStream_t stream) {
    if (dt != MSLA_F32 && dt != MSLA_F16 && dt != MSLA_BF16) return MSLA_ERR_INVALID_ARG;
    return multiscale_state_impl(qkv, w_dw, w_gpw, q_ms, kv, scratch, scratch_bytes, B, H, W, heads, head_dim,
                                 scales, n_scales, (msla_dtype)dt, stream, /*small=*/true);
}
