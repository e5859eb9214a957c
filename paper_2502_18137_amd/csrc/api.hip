// C ABI of libsparge: argument validation, workspace partition, kernel sequencing.
// Nothing here allocates device memory; every kernel goes onto the caller's stream, except that
// sparge_forward runs three passes on a second stream between a fork and a join on the caller's.  Only
// sparge_tune synchronises (it decides on the host between candidates).
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <algorithm>
#include <mutex>
#include <vector>

#include "common.hpp"

using namespace sparge;

// Scratch of sparge_predict_static: the predictor's intermediates for callers that cannot pass a workspace.
// Every device the library runs on holds its own copy at its own address; host code never uses this name as
// an address, only the pointer hipGetSymbolAddress returns for the current device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[SPARGE_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";
thread_local void* const* g_ev_start = nullptr;
thread_local void* const* g_ev_stop = nullptr;
thread_local int g_ev_n = 0, g_ev_k = 0;

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(SPARGE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

int check_desc(const sparge_desc* d, Shape* s) {
    if (!d) return fail(SPARGE_EINVAL, "desc is NULL");
    if (d->B < 1 || d->H < 1 || d->N < 1) return fail(SPARGE_EINVAL, "B, H, N must be >= 1 (got %d, %d, %d)", d->B, d->H, d->N);
    if (d->d != 64 && d->d != 128) return fail(SPARGE_EUNSUPPORTED, "head dim %d not supported (64 or 128)", d->d);
    if (d->dtype != SPARGE_F16 && d->dtype != SPARGE_BF16) return fail(SPARGE_EUNSUPPORTED, "dtype %d not supported", d->dtype);
    if (d->H > SPARGE_MAX_HEADS) return fail(SPARGE_EUNSUPPORTED, "H = %d exceeds %d", d->H, SPARGE_MAX_HEADS);
    if ((long long)d->B * d->H > 65535) return fail(SPARGE_EUNSUPPORTED, "B*H exceeds 65535");
    const int Tn = (d->N + BK - 1) / BK;
    if (Tn > SPARGE_MAX_TN) return fail(SPARGE_EUNSUPPORTED, "N = %d gives %d key blocks, more than %d", d->N, Tn, SPARGE_MAX_TN);
    if (d->stride_n < d->d || d->stride_b < 0 || d->stride_h < 0) return fail(SPARGE_EINVAL, "bad strides");
    if (d->stride_n % 8 || d->stride_h % 8 || d->stride_b % 8) return fail(SPARGE_EINVAL, "strides must be multiples of 8 elements");
    s->B = d->B; s->H = d->H; s->N = d->N; s->d = d->d; s->dtype = d->dtype;
    s->sb = d->stride_b; s->sh = d->stride_h; s->sn = d->stride_n;
    s->Tm = (d->N + BQ - 1) / BQ;
    s->Tn = Tn;
    if (d->pv_dtype != SPARGE_PV_16BIT && d->pv_dtype != SPARGE_PV_FP8)
        return fail(SPARGE_EUNSUPPORTED, "pv_dtype %d not supported", d->pv_dtype);
    s->pv_fp8 = d->pv_dtype == SPARGE_PV_FP8;
    if (d->qk_dtype != SPARGE_QK_INT8 && d->qk_dtype != SPARGE_QK_16BIT)
        return fail(SPARGE_EUNSUPPORTED, "qk_dtype %d not supported", d->qk_dtype);
    s->qk16 = d->qk_dtype == SPARGE_QK_16BIT;
    if (s->qk16 && s->pv_fp8) return fail(SPARGE_EUNSUPPORTED, "the 16-bit Q K^T product is not built with the FP8 P~V product");
    if (s->qk16 && Tn > 2048) return fail(SPARGE_EUNSUPPORTED, "the 16-bit Q K^T product takes at most 2048 key blocks (N <= 131072)");
    if (s->qk16 && (double)Tn * BK * d->stride_n * 2.0 >= 4294967296.0)
        return fail(SPARGE_EUNSUPPORTED, "the 16-bit Q K^T product needs a head's K to span less than 4 GiB");
    return SPARGE_OK;
}

// Re-tiled V: the tiles, and for the FP8 product the channel scales and maxima behind them.
struct VTiles {
    size_t scale, amax, total;
};
VTiles v_tiles_layout(const Shape& s) {
    const size_t BH = (size_t)s.B * s.H;
    VTiles v{};
    if (!s.pv_fp8) {
        v.total = BH * s.Tn * s.d * BK * sizeof(uint16_t);
        return v;
    }
    v.scale = align256(BH * s.Tn * s.d * BK);
    v.amax = v.scale + align256(BH * s.d * sizeof(float));
    v.total = v.amax + align256(BH * s.d * sizeof(uint32_t));
    return v;
}
hipError_t retile_v(const void* V, const Shape& s, void* v_tiles, hipStream_t st) {
    if (!s.pv_fp8) return launch_v_tiles(V, s, static_cast<uint16_t*>(v_tiles), st);
    const VTiles v = v_tiles_layout(s);
    char* p = static_cast<char*>(v_tiles);
    return launch_v_tiles_fp8(V, s, reinterpret_cast<unsigned char*>(p), reinterpret_cast<float*>(p + v.scale),
                              reinterpret_cast<uint32_t*>(p + v.amax), st);
}
const float* v_scale_of(const void* v_tiles, const Shape& s) {
    return s.pv_fp8 ? reinterpret_cast<const float*>(static_cast<const char*>(v_tiles) + v_tiles_layout(s).scale)
                    : nullptr;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Partition of the scratch buffer.  Every entry point uses a subset; offsets are fixed by shape.
struct Workspace {
    size_t pooled_q, ksum_t, sim_q, sim_k, k_mean, logits, Qq, Kq, q_scale, k_scale, v_tiles, mask, queue, total;
};

Workspace plan(const Shape& s, int entry) {
    const size_t BH = (size_t)s.B * s.H;
    const bool stats = entry == SPARGE_WS_QUANTIZE || entry == SPARGE_WS_PREDICT || entry == SPARGE_WS_ATTN ||
                       entry == SPARGE_WS_FORWARD;
    const bool pred = entry == SPARGE_WS_PREDICT || entry == SPARGE_WS_FORWARD;
    const bool quant_in_ws = entry == SPARGE_WS_ATTN || entry == SPARGE_WS_FORWARD;
    const bool attn = entry == SPARGE_WS_ATTN || entry == SPARGE_WS_ATTN_QUANTIZED || entry == SPARGE_WS_FORWARD;
    const bool loop = attn || entry == SPARGE_WS_ATTN_TILED;
    Workspace w{};
    size_t off = 0;
    auto take = [&](bool used, size_t bytes) { size_t o = off; if (used) off += align256(bytes); return o; };
    w.pooled_q = take(stats, BH * s.Tm * s.d * sizeof(double));
    w.ksum_t = take(stats, BH * s.Tn * s.d * sizeof(double));
    w.sim_q = take(stats, BH * s.Tm * sizeof(double));
    w.sim_k = take(stats, BH * s.Tn * sizeof(double));
    w.k_mean = take(quant_in_ws, BH * s.d * sizeof(float));
    w.logits = take(pred, BH * s.Tm * s.Tn * sizeof(double));
    w.Qq = take(quant_in_ws, BH * s.N * s.d);
    w.Kq = take(quant_in_ws, BH * s.N * s.d);
    w.q_scale = take(quant_in_ws, BH * s.Tm * sizeof(float));
    w.k_scale = take(quant_in_ws, BH * s.Tn * sizeof(float));
    w.v_tiles = take(attn, v_tiles_layout(s).total);
    w.mask = take(entry == SPARGE_WS_FORWARD, BH * s.Tm * s.Tn);
    w.queue = take(loop, ATTN_QUEUE_BYTES);  // item counters of the attention kernel's work distribution
    w.total = off ? off : 256;
    return w;
}

int check_ws(const Workspace& w, void* ws, size_t ws_bytes) {
    if (!ws) return fail(SPARGE_EINVAL, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(SPARGE_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < w.total) return fail(SPARGE_ENOSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, w.total);
    return SPARGE_OK;
}

template <typename T>
T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

int head_params(const float* src, int H, const char* name, HeadParams* out) {
    if (!src) return fail(SPARGE_EINVAL, "%s is NULL", name);
    std::memset(out, 0, sizeof(*out));
    for (int h = 0; h < H; ++h) out->v[h] = src[h];
    return SPARGE_OK;
}

int check_tau_theta(const float* tau, const float* theta, int H, HeadParams* t, HeadParams* th) {
    int rc;
    if ((rc = head_params(tau, H, "tau", t))) return rc;
    if ((rc = head_params(theta, H, "theta", th))) return rc;
    for (int h = 0; h < H; ++h) {
        if (!(tau[h] > 0.f && tau[h] <= 1.f)) return fail(SPARGE_EINVAL, "tau[%d] = %g outside (0,1]", h, tau[h]);
        if (std::isnan(theta[h])) return fail(SPARGE_EINVAL, "theta[%d] is NaN", h);
    }
    return SPARGE_OK;
}

int check_lambda(const float* lambda, int H, HeadParams* l) {
    int rc;
    if ((rc = head_params(lambda, H, "lambda", l))) return rc;
    for (int h = 0; h < H; ++h)
        if (!(lambda[h] < 0.f)) return fail(SPARGE_EINVAL, "lambda[%d] = %g must be < 0", h, lambda[h]);
    return SPARGE_OK;
}

// Block statistics of Q and K, Q quantization, K mean, K quantization (any output may be skipped).
// A second stream per device (default priority) with the two events of a fork and join.  The forward
// pass puts the passes nobody waits for early (K mean, K quantization, V tiles: bandwidth-bound) there,
// beside the block predictor (fp64 matrix products and a sort: neither bandwidth-bound), and joins before
// the attention kernel.  Created on first use, kept until the process ends; no second stream (creation
// failed, or more devices than slots) means everything runs on the caller's stream.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool tried = false;
};
constexpr int MAX_DEVICES = 64;
SideStream g_side[MAX_DEVICES];
std::mutex g_side_mutex;

// (call with g_side_mutex held, and keep it until the join is enqueued: the events are shared)
SideStream* side_stream() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    SideStream& x = g_side[dev];
    if (!x.tried) {
        x.tried = true;
        hipStream_t st = nullptr;
        hipEvent_t a = nullptr, b = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&a, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&b, hipEventDisableTiming) == hipSuccess) {
            x.stream = st, x.fork = a, x.join = b;
        } else {
            (void)hipGetLastError();  // not an error of the call that asked
        }
    }
    return x.stream ? &x : nullptr;
}

// Device address of `scratch` on the current device: looked up once per device, with that device current.
void* g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;
int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SPARGE_EUNSUPPORTED, "device %d: more devices than the library tracks", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SPARGE_OK;
}

int run_stats_and_quant(const void* Q, const void* K, const Shape& s, double* pooled_q, double* ksum_t,
                        double* sim_q, double* sim_k, int8_t* Qq, float* q_scale, int8_t* Kq, float* k_scale,
                        float* k_mean, hipStream_t st) {
    hipError_t e;
    if ((e = launch_block_stats_q(Q, s, pooled_q, sim_q, Qq, q_scale, st)) != hipSuccess) return hip_fail(e, "block_stats_q");
    if ((e = launch_block_stats_k(K, s, ksum_t, sim_k, st)) != hipSuccess) return hip_fail(e, "block_stats_k");
    if (Kq) {
        if ((e = launch_k_mean(ksum_t, s, k_mean, st)) != hipSuccess) return hip_fail(e, "k_mean");
        if ((e = launch_quant_k(K, s, k_mean, Kq, k_scale, st)) != hipSuccess) return hip_fail(e, "quant_k");
    }
    return SPARGE_OK;
}

int run_predict(const Shape& s, void* ws, const Workspace& w, const HeadParams& tau, const HeadParams& theta,
                float sm_scale, int causal, uint8_t* mask, hipStream_t st) {
    hipError_t e;
    if ((e = launch_logits(at<double>(ws, w.pooled_q), at<double>(ws, w.ksum_t), s, sm_scale,
                           at<double>(ws, w.logits), st)) != hipSuccess) return hip_fail(e, "logits");
    if ((e = launch_topcdf(at<double>(ws, w.logits), at<double>(ws, w.sim_q), at<double>(ws, w.sim_k), s, tau,
                           theta, causal, mask, st)) != hipSuccess) return hip_fail(e, "topcdf");
    return SPARGE_OK;
}

// The attention launch, bracketed by the caller's timing events when some are installed.
int timed_attn(const void* Qq, const void* Kq, const float* q_scale, const float* k_scale,
               const void* v_tiles, const Shape& s, const uint8_t* mask, const HeadParams& lam, float sm_scale,
               int causal, void* O, uint64_t* stats, unsigned int* queue, hipStream_t st) {
    const bool timed = g_ev_start && g_ev_k < g_ev_n;
    hipError_t e;
    if (stats && (e = launch_zero_stats(reinterpret_cast<unsigned long long*>(stats), s.B * s.H * 4, st)) != hipSuccess)
        return hip_fail(e, "zero stats");
    if (timed && (e = hipEventRecord(static_cast<hipEvent_t>(g_ev_start[g_ev_k]), st)) != hipSuccess)
        return hip_fail(e, "record start event");
    if ((e = launch_attn(Qq, Kq, q_scale, k_scale, v_tiles, v_scale_of(v_tiles, s), s, mask, lam, sm_scale, causal, O,
                         reinterpret_cast<unsigned long long*>(stats), queue, st)) != hipSuccess)
        return hip_fail(e, "attn");
    if (timed) {
        if ((e = hipEventRecord(static_cast<hipEvent_t>(g_ev_stop[g_ev_k]), st)) != hipSuccess)
            return hip_fail(e, "record stop event");
        ++g_ev_k;
    }
    return SPARGE_OK;
}

int run_attn(const void* Qq, const void* Kq, const float* q_scale, const float* k_scale, const void* V,
             const Shape& s, void* v_tiles, const uint8_t* mask, const HeadParams& lam, float sm_scale,
             int causal, void* O, uint64_t* stats, unsigned int* queue, hipStream_t st) {
    hipError_t e;
    if ((e = retile_v(V, s, v_tiles, st)) != hipSuccess) return hip_fail(e, "v_tiles");
    return timed_attn(Qq, Kq, q_scale, k_scale, v_tiles, s, mask, lam, sm_scale, causal, O, stats, queue, st);
}

}  // namespace

extern "C" {

const char* sparge_last_error(void) { return g_err; }

int sparge_version(void) { return 100; }

int sparge_workspace_bytes(const sparge_desc* desc, int entry, size_t* bytes) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!bytes) return fail(SPARGE_EINVAL, "bytes is NULL");
    if (entry < SPARGE_WS_QUANTIZE || entry > SPARGE_WS_ATTN_TILED) return fail(SPARGE_EINVAL, "unknown entry %d", entry);
    *bytes = plan(s, entry).total;
    return SPARGE_OK;
}

int sparge_quantize(const void* Q, const void* K, const sparge_desc* desc, int8_t* Qq, int8_t* Kq,
                    float* q_scale, float* k_scale, float* k_mean, void* ws, size_t ws_bytes, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!Q || !K || !Qq || !Kq || !q_scale || !k_scale || !k_mean) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(Q) || misaligned(K) || misaligned(Qq) || misaligned(Kq) || misaligned(k_mean))
        return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    const Workspace w = plan(s, SPARGE_WS_QUANTIZE);
    if ((rc = check_ws(w, ws, ws_bytes))) return rc;
    return run_stats_and_quant(Q, K, s, at<double>(ws, w.pooled_q), at<double>(ws, w.ksum_t), at<double>(ws, w.sim_q),
                               at<double>(ws, w.sim_k), Qq, q_scale, Kq, k_scale, k_mean,
                               static_cast<hipStream_t>(hip_stream));
}

int sparge_predict(const void* Q, const void* K, const sparge_desc* desc, const float* tau, const float* theta,
                   float sm_scale, int causal, uint8_t* mask, double* sim_q, double* sim_k, void* ws,
                   size_t ws_bytes, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!Q || !K || !mask) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(Q) || misaligned(K)) return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    HeadParams t, th;
    if ((rc = check_tau_theta(tau, theta, s.H, &t, &th))) return rc;
    const Workspace w = plan(s, SPARGE_WS_PREDICT);
    if ((rc = check_ws(w, ws, ws_bytes))) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if ((rc = run_stats_and_quant(Q, K, s, at<double>(ws, w.pooled_q), at<double>(ws, w.ksum_t),
                                  at<double>(ws, w.sim_q), at<double>(ws, w.sim_k), nullptr, nullptr, nullptr,
                                  nullptr, nullptr, st))) return rc;
    if ((rc = run_predict(s, ws, w, t, th, sm_scale, causal, mask, st))) return rc;
    const size_t BH = (size_t)s.B * s.H;
    hipError_t e;
    if (sim_q && (e = hipMemcpyAsync(sim_q, at<double>(ws, w.sim_q), BH * s.Tm * sizeof(double),
                                     hipMemcpyDeviceToDevice, st)) != hipSuccess) return hip_fail(e, "copy sim_q");
    if (sim_k && (e = hipMemcpyAsync(sim_k, at<double>(ws, w.sim_k), BH * s.Tn * sizeof(double),
                                     hipMemcpyDeviceToDevice, st)) != hipSuccess) return hip_fail(e, "copy sim_k");
    return SPARGE_OK;
}

int sparge_predict_static(const void* Q, const void* K, const sparge_desc* desc, const float* tau,
                          const float* theta, float sm_scale, int causal, uint8_t* mask, double* sim_q,
                          double* sim_k, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    const size_t need = plan(s, SPARGE_WS_PREDICT).total;
    if (need > SPARGE_STATIC_SCRATCH_BYTES)
        return fail(SPARGE_ENOSPACE, "sparge_predict_static: this shape needs %zu bytes of scratch, the static buffer has %zu; "
                    "use sparge_predict with a workspace", need, (size_t)SPARGE_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    return sparge_predict(Q, K, desc, tau, theta, sm_scale, causal, mask, sim_q, sim_k, ws,
                          SPARGE_STATIC_SCRATCH_BYTES, hip_stream);
}

int sparge_item_order(const sparge_desc* desc, int causal, int32_t* order) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!order) return fail(SPARGE_EINVAL, "order is NULL");
    const int n_work = s.B * s.H * s.Tm, per_range = (n_work + 7) / 8;
    int n = 0;
    for (int y = 0; y < 8; ++y) {
        const int len = std::min(per_range, n_work - y * per_range);
        for (int p = 0; p < len; ++p) {
            const int g = range_item(y * per_range, len, p, s.Tm, causal != 0);
            const int q = g % s.Tm;
            order[n++] = g - q + (causal ? s.Tm - 1 - q : q);
        }
    }
    return SPARGE_OK;
}

int sparge_mask_to_lut(const uint8_t* mask, const sparge_desc* desc, int32_t* lut, int32_t* lut_count, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!mask || !lut || !lut_count) return fail(SPARGE_EINVAL, "NULL argument");
    if (reinterpret_cast<uintptr_t>(lut) % 4 || reinterpret_cast<uintptr_t>(lut_count) % 4)
        return fail(SPARGE_EINVAL, "lut and lut_count must be 4-byte aligned");
    hipError_t e = launch_mask_lut(mask, s, lut, lut_count, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARGE_OK : hip_fail(e, "mask_lut");
}

int sparge_attn_quantized(const int8_t* Qq, const int8_t* Kq, const float* q_scale, const float* k_scale,
                          const void* V, const sparge_desc* desc, const uint8_t* mask, const float* lambda,
                          float sm_scale, int causal, void* O, uint64_t* stats, void* ws, size_t ws_bytes,
                          void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!Qq || !Kq || !q_scale || !k_scale || !V || !O) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(Qq) || misaligned(Kq) || misaligned(V) || misaligned(O))
        return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    HeadParams lam;
    if ((rc = check_lambda(lambda, s.H, &lam))) return rc;
    const Workspace w = plan(s, SPARGE_WS_ATTN_QUANTIZED);
    if ((rc = check_ws(w, ws, ws_bytes))) return rc;
    return run_attn(Qq, Kq, q_scale, k_scale, V, s, at<char>(ws, w.v_tiles), mask, lam, sm_scale, causal, O,
                    stats, at<unsigned int>(ws, w.queue), static_cast<hipStream_t>(hip_stream));
}

int sparge_v_tiles_bytes(const sparge_desc* desc, size_t* bytes) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!bytes) return fail(SPARGE_EINVAL, "bytes is NULL");
    *bytes = v_tiles_layout(s).total;
    return SPARGE_OK;
}

int sparge_v_tiles(const void* V, const sparge_desc* desc, void* v_tiles, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!V || !v_tiles) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(V) || misaligned(v_tiles)) return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    hipError_t e = retile_v(V, s, v_tiles, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARGE_OK : hip_fail(e, "v_tiles");
}

int sparge_attn_tiled(const int8_t* Qq, const int8_t* Kq, const float* q_scale, const float* k_scale,
                      const void* v_tiles, const sparge_desc* desc, const uint8_t* mask, const float* lambda,
                      float sm_scale, int causal, void* O, uint64_t* stats, void* ws, size_t ws_bytes,
                      void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!Qq || !Kq || !q_scale || !k_scale || !v_tiles || !O) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(Qq) || misaligned(Kq) || misaligned(v_tiles) || misaligned(O))
        return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    HeadParams lam;
    if ((rc = check_lambda(lambda, s.H, &lam))) return rc;
    const Workspace w = plan(s, SPARGE_WS_ATTN_TILED);
    if ((rc = check_ws(w, ws, ws_bytes))) return rc;
    return timed_attn(Qq, Kq, q_scale, k_scale, v_tiles, s, mask, lam, sm_scale, causal,
                      O, stats, at<unsigned int>(ws, w.queue), static_cast<hipStream_t>(hip_stream));
}

int sparge_attn(const void* Q, const void* K, const void* V, const sparge_desc* desc, const uint8_t* mask,
                const float* lambda, float sm_scale, int causal, void* O, uint64_t* stats, void* ws,
                size_t ws_bytes, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!Q || !K || !V || !O) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    HeadParams lam;
    if ((rc = check_lambda(lambda, s.H, &lam))) return rc;
    const Workspace w = plan(s, SPARGE_WS_ATTN);
    if ((rc = check_ws(w, ws, ws_bytes))) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (s.qk16)  // the products run on Q and K as they are: nothing to quantize
        return run_attn(Q, K, nullptr, nullptr, V, s, at<char>(ws, w.v_tiles), mask, lam, sm_scale, causal, O, stats,
                        at<unsigned int>(ws, w.queue), st);
    if ((rc = run_stats_and_quant(Q, K, s, at<double>(ws, w.pooled_q), at<double>(ws, w.ksum_t),
                                  at<double>(ws, w.sim_q), at<double>(ws, w.sim_k), at<int8_t>(ws, w.Qq),
                                  at<float>(ws, w.q_scale), at<int8_t>(ws, w.Kq), at<float>(ws, w.k_scale),
                                  at<float>(ws, w.k_mean), st))) return rc;
    return run_attn(at<int8_t>(ws, w.Qq), at<int8_t>(ws, w.Kq), at<float>(ws, w.q_scale), at<float>(ws, w.k_scale),
                    V, s, at<char>(ws, w.v_tiles), mask, lam, sm_scale, causal, O, stats, at<unsigned int>(ws, w.queue), st);
}

int sparge_forward(const void* Q, const void* K, const void* V, const sparge_desc* desc, const float* tau,
                   const float* theta, const float* lambda, float sm_scale, int causal, void* O,
                   uint8_t* mask_out, uint64_t* stats, void* ws, size_t ws_bytes, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!Q || !K || !V || !O) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    HeadParams t, th, lam;
    if ((rc = check_tau_theta(tau, theta, s.H, &t, &th))) return rc;
    if ((rc = check_lambda(lambda, s.H, &lam))) return rc;
    const Workspace w = plan(s, SPARGE_WS_FORWARD);
    if ((rc = check_ws(w, ws, ws_bytes))) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool q8 = !s.qk16;  // the 16-bit product needs the block statistics only
    uint8_t* mask = mask_out ? mask_out : at<uint8_t>(ws, w.mask);
    const void* Qa = q8 ? static_cast<const void*>(at<int8_t>(ws, w.Qq)) : Q;
    const void* Ka = q8 ? static_cast<const void*>(at<int8_t>(ws, w.Kq)) : K;
    const float* qsc = q8 ? at<float>(ws, w.q_scale) : nullptr;
    const float* ksc = q8 ? at<float>(ws, w.k_scale) : nullptr;
    std::lock_guard<std::mutex> lock(g_side_mutex);
    SideStream* side = side_stream();
    if (!side) {
        if ((rc = run_stats_and_quant(Q, K, s, at<double>(ws, w.pooled_q), at<double>(ws, w.ksum_t),
                                      at<double>(ws, w.sim_q), at<double>(ws, w.sim_k), q8 ? at<int8_t>(ws, w.Qq) : nullptr,
                                      q8 ? at<float>(ws, w.q_scale) : nullptr, q8 ? at<int8_t>(ws, w.Kq) : nullptr,
                                      at<float>(ws, w.k_scale), at<float>(ws, w.k_mean), st))) return rc;
        if ((rc = run_predict(s, ws, w, t, th, sm_scale, causal, mask, st))) return rc;
        return run_attn(Qa, Ka, qsc, ksc, V, s, at<char>(ws, w.v_tiles), mask, lam, sm_scale, causal, O, stats,
                        at<unsigned int>(ws, w.queue), st);
    }
    // caller's stream: block statistics (+ Q quantization) -> fork -> predictor -> join -> attention
    // second stream:                                  fork -> V tiles, K mean, K quantization -> join
    hipError_t e;
    if ((e = launch_block_stats_q(Q, s, at<double>(ws, w.pooled_q), at<double>(ws, w.sim_q),
                                  q8 ? at<int8_t>(ws, w.Qq) : nullptr, q8 ? at<float>(ws, w.q_scale) : nullptr, st)) != hipSuccess)
        return hip_fail(e, "block_stats_q");
    if ((e = launch_block_stats_k(K, s, at<double>(ws, w.ksum_t), at<double>(ws, w.sim_k), st)) != hipSuccess)
        return hip_fail(e, "block_stats_k");
    if ((e = hipEventRecord(side->fork, st)) != hipSuccess) return hip_fail(e, "record fork");
    if ((e = hipStreamWaitEvent(side->stream, side->fork, 0)) != hipSuccess) return hip_fail(e, "wait fork");
    // from here on the second stream is joined whatever happens, so that a capture of the caller's stream can end
    int rc_side = SPARGE_OK;
    // V tiles first: they need LDS, which the logits kernel beside them leaves free and TopCdf does not
    if ((e = retile_v(V, s, at<char>(ws, w.v_tiles), side->stream)) != hipSuccess) rc_side = hip_fail(e, "v_tiles");
    if (q8 && !rc_side) {
        if ((e = launch_k_mean(at<double>(ws, w.ksum_t), s, at<float>(ws, w.k_mean), side->stream)) != hipSuccess)
            rc_side = hip_fail(e, "k_mean");
        else if ((e = launch_quant_k(K, s, at<float>(ws, w.k_mean), at<int8_t>(ws, w.Kq), at<float>(ws, w.k_scale),
                                     side->stream)) != hipSuccess)
            rc_side = hip_fail(e, "quant_k");
    }
    rc = rc_side ? SPARGE_OK : run_predict(s, ws, w, t, th, sm_scale, causal, mask, st);
    if ((e = hipEventRecord(side->join, side->stream)) != hipSuccess) return hip_fail(e, "record join");
    if ((e = hipStreamWaitEvent(st, side->join, 0)) != hipSuccess) return hip_fail(e, "wait join");
    if (rc_side) return rc_side;
    if (rc) return rc;
    return timed_attn(Qa, Ka, qsc, ksc, at<char>(ws, w.v_tiles), s, mask, lam, sm_scale, causal, O, stats,
                      at<unsigned int>(ws, w.queue), st);
}

int sparge_rel_l1(const void* O, const void* O_ref, const sparge_desc* desc, double* out, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!O || !O_ref || !out) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (misaligned(O) || misaligned(O_ref)) return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    hipError_t e = launch_rel_l1(O, O_ref, s, out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARGE_OK : hip_fail(e, "rel_l1");
}

namespace {

// Workspace of the hyper-parameter search: per input a forward workspace and the full-attention output,
// then one output buffer, the error sums and the counters.
struct TuneWs {
    size_t fwd_bytes, out_bytes, per_input, o_cur, metrics, stats, total;
};
TuneWs tune_layout(const Shape& s, int n_inputs) {
    TuneWs t{};
    t.fwd_bytes = align256(plan(s, SPARGE_WS_FORWARD).total);
    const size_t span = (size_t)(s.B - 1) * s.sb + (size_t)(s.H - 1) * s.sh + (size_t)(s.N - 1) * s.sn + s.d;
    t.out_bytes = align256(span * sizeof(uint16_t));
    t.per_input = t.fwd_bytes + t.out_bytes;
    t.o_cur = t.per_input * n_inputs;
    t.metrics = t.o_cur + t.out_bytes;
    t.stats = t.metrics + align256((size_t)s.B * s.H * 2 * sizeof(double));
    t.total = t.stats + align256((size_t)s.B * s.H * 4 * sizeof(uint64_t));
    return t;
}

}  // namespace

int sparge_tune_workspace_bytes(const sparge_desc* desc, int n_inputs, size_t* bytes) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (n_inputs < 1 || !bytes) return fail(SPARGE_EINVAL, "n_inputs must be >= 1 and bytes not NULL");
    *bytes = tune_layout(s, n_inputs).total;
    return SPARGE_OK;
}

int sparge_tune(const void* const* Q, const void* const* K, const void* const* V, int n_inputs,
                const sparge_desc* desc, const float* tau_grid, int n_tau, const float* theta_grid, int n_theta,
                const float* lambda_grid, int n_lambda, float l1, float l2, float sm_scale, int causal,
                float* tau, float* theta, float* lambda, double* sparsity, double* l1_out, double* stage1,
                double* stage2, void* ws, size_t ws_bytes, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (n_inputs < 1 || !Q || !K || !V) return fail(SPARGE_EINVAL, "no inputs");
    if (n_tau < 1 || n_theta < 1 || n_lambda < 0 || !tau_grid || !theta_grid || (n_lambda && !lambda_grid))
        return fail(SPARGE_EINVAL, "empty tau/theta grid or missing lambda grid");
    if (!tau || !theta || !lambda) return fail(SPARGE_EINVAL, "result arrays are NULL");
    for (int n = 0; n < n_inputs; ++n) {
        if (!Q[n] || !K[n] || !V[n]) return fail(SPARGE_EINVAL, "input %d has a NULL tensor", n);
        if (misaligned(Q[n]) || misaligned(K[n]) || misaligned(V[n]))
            return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    }
    for (int a = 0; a < n_tau; ++a)
        if (!(tau_grid[a] > 0.f && tau_grid[a] <= 1.f)) return fail(SPARGE_EINVAL, "tau_grid[%d] outside (0,1]", a);
    for (int b = 0; b < n_theta; ++b)
        if (std::isnan(theta_grid[b])) return fail(SPARGE_EINVAL, "theta_grid[%d] is NaN", b);
    for (int c = 0; c < n_lambda; ++c)
        if (!(lambda_grid[c] < 0.f)) return fail(SPARGE_EINVAL, "lambda_grid[%d] must be < 0", c);
    const TuneWs t = tune_layout(s, n_inputs);
    if (!ws) return fail(SPARGE_EINVAL, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(SPARGE_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < t.total) return fail(SPARGE_ENOSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, t.total);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Workspace w = plan(s, SPARGE_WS_FORWARD);
    const int BH = s.B * s.H, H = s.H;
    auto fwd = [&](int n) { return static_cast<void*>(static_cast<char*>(ws) + t.per_input * n); };
    auto o_ref = [&](int n) { return static_cast<void*>(static_cast<char*>(ws) + t.per_input * n + t.fwd_bytes); };
    void* o_cur = at<char>(ws, t.o_cur);
    double* d_metrics = at<double>(ws, t.metrics);
    uint64_t* d_stats = at<uint64_t>(ws, t.stats);
    hipError_t e;

    // per input, once: block statistics, quantization, V tiles, and the full attention it is measured against
    HeadParams off;
    std::memset(&off, 0, sizeof(off));
    for (int h = 0; h < H; ++h) off.v[h] = -INFINITY;
    for (int n = 0; n < n_inputs; ++n) {
        void* f = fwd(n);
        if ((rc = run_stats_and_quant(Q[n], K[n], s, at<double>(f, w.pooled_q), at<double>(f, w.ksum_t),
                                      at<double>(f, w.sim_q), at<double>(f, w.sim_k), at<int8_t>(f, w.Qq),
                                      at<float>(f, w.q_scale), at<int8_t>(f, w.Kq), at<float>(f, w.k_scale),
                                      at<float>(f, w.k_mean), st))) return rc;
        if ((rc = run_attn(at<int8_t>(f, w.Qq), at<int8_t>(f, w.Kq), at<float>(f, w.q_scale), at<float>(f, w.k_scale),
                           V[n], s, at<char>(f, w.v_tiles), nullptr, off, sm_scale, causal, o_ref(n), nullptr,
                           at<unsigned int>(f, w.queue), st)))
            return rc;
    }

    std::vector<double> h_metrics(BH * 2);
    std::vector<uint64_t> h_stats(BH * 4);
    // one setting on every input: per head the mean sparsity and the worst relative L1
    auto evaluate = [&](const HeadParams& tp, const HeadParams& thp, const HeadParams& lp, double* sp, double* err) -> int {
        for (int h = 0; h < H; ++h) { sp[h] = 0.0; err[h] = 0.0; }
        for (int n = 0; n < n_inputs; ++n) {
            void* f = fwd(n);
            int r;
            if ((r = run_predict(s, f, w, tp, thp, sm_scale, causal, at<uint8_t>(f, w.mask), st))) return r;
            if ((r = timed_attn(at<int8_t>(f, w.Qq), at<int8_t>(f, w.Kq), at<float>(f, w.q_scale),
                                at<float>(f, w.k_scale), at<char>(f, w.v_tiles), s, at<uint8_t>(f, w.mask), lp,
                                sm_scale, causal, o_cur, d_stats, at<unsigned int>(f, w.queue), st))) return r;
            if ((e = launch_rel_l1(o_cur, o_ref(n), s, d_metrics, st)) != hipSuccess) return hip_fail(e, "rel_l1");
            if ((e = hipMemcpyAsync(h_metrics.data(), d_metrics, BH * 2 * sizeof(double), hipMemcpyDeviceToHost, st)) != hipSuccess)
                return hip_fail(e, "copy error sums");
            if ((e = hipMemcpyAsync(h_stats.data(), d_stats, BH * 4 * sizeof(uint64_t), hipMemcpyDeviceToHost, st)) != hipSuccess)
                return hip_fail(e, "copy counters");
            if ((e = hipStreamSynchronize(st)) != hipSuccess) return hip_fail(e, "synchronize");
            for (int h = 0; h < H; ++h) {
                double num = 0.0, den = 0.0;
                uint64_t c[4] = {0, 0, 0, 0};
                for (int b = 0; b < s.B; ++b) {
                    num += h_metrics[(b * H + h) * 2 + 0];
                    den += h_metrics[(b * H + h) * 2 + 1];
                    for (int q = 0; q < 4; ++q) c[q] += h_stats[(b * H + h) * 4 + q];
                }
                sp[h] += 1.0 - 0.5 * ((double)c[0] / (double)c[2] + (double)c[1] / (double)c[3]);
                err[h] = std::fmax(err[h], num / den);
            }
        }
        for (int h = 0; h < H; ++h) sp[h] /= n_inputs;
        return SPARGE_OK;
    };

    // stage 1: the (tau, theta) grid with the lambda test off
    const int n1 = n_tau * n_theta;
    std::vector<double> t1((size_t)n1 * H * 2), sp(H), err(H);
    HeadParams tp, thp, lp;
    std::memset(&tp, 0, sizeof(tp));
    std::memset(&thp, 0, sizeof(thp));
    for (int a = 0; a < n_tau; ++a)
        for (int b = 0; b < n_theta; ++b) {
            for (int h = 0; h < H; ++h) { tp.v[h] = tau_grid[a]; thp.v[h] = theta_grid[b]; }
            if ((rc = evaluate(tp, thp, off, sp.data(), err.data()))) return rc;
            for (int h = 0; h < H; ++h) {
                t1[((size_t)(a * n_theta + b) * H + h) * 2 + 0] = sp[h];
                t1[((size_t)(a * n_theta + b) * H + h) * 2 + 1] = err[h];
            }
        }
    std::vector<double> best_sp(H), best_err(H);
    for (int h = 0; h < H; ++h) {
        int best = -1;
        for (int k = 0; k < n1; ++k) {  // the sparsest admissible pair; the earlier one of equals
            const double ks = t1[((size_t)k * H + h) * 2], ke = t1[((size_t)k * H + h) * 2 + 1];
            if (ke < (double)l1 && (best < 0 || ks > t1[((size_t)best * H + h) * 2])) best = k;
        }
        if (best < 0) {                 // nothing admissible: the most accurate pair
            best = 0;
            for (int k = 1; k < n1; ++k)
                if (t1[((size_t)k * H + h) * 2 + 1] < t1[((size_t)best * H + h) * 2 + 1]) best = k;
        }
        tau[h] = tau_grid[best / n_theta];
        theta[h] = theta_grid[best % n_theta];
        lambda[h] = -INFINITY;
        best_sp[h] = t1[((size_t)best * H + h) * 2];
        best_err[h] = t1[((size_t)best * H + h) * 2 + 1];
        tp.v[h] = tau[h];
        thp.v[h] = theta[h];
    }
    if (stage1) std::memcpy(stage1, t1.data(), t1.size() * sizeof(double));

    // stage 2: the lambda grid at each head's own (tau, theta)
    std::memset(&lp, 0, sizeof(lp));
    for (int c = 0; c < n_lambda; ++c) {
        for (int h = 0; h < H; ++h) lp.v[h] = lambda_grid[c];
        if ((rc = evaluate(tp, thp, lp, sp.data(), err.data()))) return rc;
        for (int h = 0; h < H; ++h) {
            if (stage2) { stage2[((size_t)c * H + h) * 2] = sp[h]; stage2[((size_t)c * H + h) * 2 + 1] = err[h]; }
            if (err[h] < (double)l2 && sp[h] > best_sp[h]) {
                lambda[h] = lambda_grid[c];
                best_sp[h] = sp[h];
                best_err[h] = err[h];
            }
        }
    }
    for (int h = 0; h < H; ++h) {
        if (sparsity) sparsity[h] = best_sp[h];
        if (l1_out) l1_out[h] = best_err[h];
    }
    return SPARGE_OK;
}

int sparge_hilbert_order(int T, int H, int W, int32_t* perm) {
    if (T < 1 || H < 1 || W < 1) return fail(SPARGE_EINVAL, "grid dimensions must be >= 1 (got %d, %d, %d)", T, H, W);
    if (T > 1024 || H > 1024 || W > 1024 || (long long)T * H * W > (1ll << 30))
        return fail(SPARGE_EUNSUPPORTED, "grid %d x %d x %d too large", T, H, W);
    if (!perm) return fail(SPARGE_EINVAL, "perm is NULL");
    hilbert_order_host(T, H, W, perm);
    return SPARGE_OK;
}

int sparge_permute_tokens(const void* src, const sparge_desc* desc, const int32_t* perm, int L, int offset,
                          int inverse, void* dst, void* hip_stream) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc) return rc;
    if (!src || !dst || !perm) return fail(SPARGE_EINVAL, "NULL tensor argument");
    if (src == dst) return fail(SPARGE_EINVAL, "src and dst must not be the same tensor");
    if (misaligned(src) || misaligned(dst)) return fail(SPARGE_EINVAL, "tensor pointers must be 16-byte aligned");
    if (L < 0 || offset < 0 || (long long)offset + L > s.N)
        return fail(SPARGE_EINVAL, "tokens [%d, %d) do not lie inside N = %d", offset, offset + L, s.N);
    hipError_t e = launch_permute_tokens(src, s, perm, L, offset, inverse, dst, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SPARGE_OK : hip_fail(e, "permute_tokens");
}

int sparge_set_timing_events(void* const* starts, void* const* stops, int n) {
    if (n < 0) return fail(SPARGE_EINVAL, "n must be >= 0");
    if (n > 0 && (!starts || !stops)) return fail(SPARGE_EINVAL, "event arrays are NULL");
    g_ev_start = n ? starts : nullptr;
    g_ev_stop = n ? stops : nullptr;
    g_ev_n = n;
    g_ev_k = 0;
    return SPARGE_OK;
}

}  // extern "C"
