// A client of libhac's C ABI that uses nothing but include/hac.h and the HIP runtime (no Python,
// no torch): it makes a small pruned, weight-shared matrix, encodes it, copies blob and batch to
// the device with hipMalloc / hipMemcpy, calls hac_dot / shac_dot on a stream of its own and a
// two-layer hac_forward on a network blob, and compares with plain double-precision loops on the
// host.  Built as a shared library so that the GPU tests can call abi_client_run() through ctypes;
// returns 0 when everything agrees, else a step number, with a message in `msg`.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/hac.h"

namespace {

struct Lcg {
    uint64_t s;
    double next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (double)(s >> 11) / 9007199254740992.0; }
};

std::vector<float> make_layer(Lcg& r, int n, int m, double density, int k)
{
    std::vector<float> W((size_t)n * m, 0.0f);
    for (auto& w : W)
        if (r.next() < density) {
            const int i = (int)(r.next() * k);
            w = (float)(i - k / 2) * 0.03125f + 0.015625f;          // k representatives, none 0
        }
    return W;
}

struct DevBuf {
    void* p = nullptr;
    explicit DevBuf(size_t bytes) { if (hipMalloc(&p, bytes ? bytes : 256) != hipSuccess) p = nullptr; }
    ~DevBuf() { if (p) (void)hipFree(p); }
};

// |Y - X.W| <= tol * |X|.|W| element by element
bool close_to_dense(const std::vector<float>& Y, const std::vector<float>& X, const std::vector<float>& W,
                    int B, int n, int m, double tol)
{
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < m; ++j) {
            double ref = 0.0, scale = 0.0;
            for (int i = 0; i < n; ++i) {
                const double t = (double)X[(size_t)b * n + i] * (double)W[(size_t)i * m + j];
                ref += t; scale += std::fabs(t);
            }
            if (std::fabs((double)Y[(size_t)b * m + j] - ref) > tol * scale + 1e-30) return false;
        }
    return true;
}

} // namespace

#define FAIL(step, ...) do { std::snprintf(msg, msg_len, __VA_ARGS__); return step; } while (0)

extern "C" int abi_client_run(char* msg, size_t msg_len)
{
    if (msg && msg_len) msg[0] = 0;
    Lcg rng = { 12345 };
    const int n = 700, m = 150, B = 37;
    std::vector<float> W = make_layer(rng, n, m, 0.05, 20);
    std::vector<float> X((size_t)B * n);
    for (auto& x : X) { const double u = rng.next() * 2.0 - 0.7; x = u > 0 ? (float)u : 0.0f; }
    hipStream_t stream;
    if (hipStreamCreate(&stream) != hipSuccess) FAIL(1, "hipStreamCreate failed");

    for (int fmt = 0; fmt < 3; ++fmt) {                          // HAC, sHAC, sHAC with Rice-coded gaps
        void* blob = nullptr; size_t bytes = 0;
        hac_opts_t o; std::memset(&o, 0, sizeof o);
        o.ri_coding = fmt == 2 ? HAC_RI_RICE : HAC_RI_FIELDS;
        int rc = fmt == 0 ? hac_encode(W.data(), n, m, m, &o, &blob, &bytes) : shac_encode(W.data(), n, m, m, &o, &blob, &bytes);
        if (rc) FAIL(10 + fmt, "encode: %s", hac_strerror(rc));
        if ((rc = hac_validate(blob, bytes, 1))) FAIL(20 + fmt, "validate: %s", hac_strerror(rc));
        hac_desc_t desc;
        if ((rc = hac_describe(blob, bytes, &desc))) FAIL(30 + fmt, "describe: %s", hac_strerror(rc));
        for (int Bc : { 1, B }) {
            const size_t ws_bytes = hac_workspace_bytes(&desc, Bc);
            DevBuf d_blob(bytes), d_X(4ull * Bc * n), d_Y(4ull * Bc * m), d_ws(ws_bytes);
            if (!d_blob.p || !d_X.p || !d_Y.p || !d_ws.p) FAIL(40 + fmt, "hipMalloc failed");
            if (hipMemcpy(d_blob.p, blob, bytes, hipMemcpyHostToDevice) != hipSuccess ||
                hipMemcpy(d_X.p, X.data(), 4ull * Bc * n, hipMemcpyHostToDevice) != hipSuccess) FAIL(50 + fmt, "hipMemcpy failed");
            rc = (fmt == 0 ? hac_dot : shac_dot)(&desc, d_blob.p, static_cast<const float*>(d_X.p), Bc, n,
                                                 static_cast<float*>(d_Y.p), m, d_ws.p, ws_bytes, nullptr, stream);
            if (rc) FAIL(60 + fmt, "dot: %s (hip %d)", hac_strerror(rc), hac_last_hip_error());
            if (hipStreamSynchronize(stream) != hipSuccess) FAIL(70 + fmt, "stream failed");
            std::vector<float> Y((size_t)Bc * m);
            if (hipMemcpy(Y.data(), d_Y.p, 4ull * Bc * m, hipMemcpyDeviceToHost) != hipSuccess) FAIL(80 + fmt, "copy back failed");
            if (!close_to_dense(Y, X, W, Bc, n, m, 1e-5)) FAIL(90 + fmt, "format %d, B = %d: result off", fmt, Bc);
        }
        hac_free(blob);
    }

    // two layers with one dictionary, bias and max(., 0) after the first
    const int m2 = 40;
    std::vector<float> W2 = make_layer(rng, m, m2, 0.2, 20);
    std::vector<float> bias((size_t)m);
    for (auto& v : bias) v = (float)(rng.next() - 0.5) * 0.1f;
    const uint32_t formats[2] = { HAC_FORMAT_SHAC, HAC_FORMAT_HAC };
    const float* Ws[2] = { W.data(), W2.data() };
    const int64_t ns[2] = { n, m }, ms[2] = { m, m2 };
    void* net = nullptr; size_t net_bytes = 0;
    int rc = hac_net_encode(2, formats, Ws, ns, ms, ms, nullptr, &net, &net_bytes);
    if (rc) FAIL(100, "net encode: %s", hac_strerror(rc));
    if ((rc = hac_net_validate(net, net_bytes, 1))) FAIL(101, "net validate: %s", hac_strerror(rc));
    hac_desc_t d0, d1;
    if (hac_net_layer(net, net_bytes, 0, &d0) || hac_net_layer(net, net_bytes, 1, &d1)) FAIL(102, "net layer");
    DevBuf d_net(net_bytes), d_X(4ull * B * n), d_Y(4ull * B * m2), d_bias(4ull * m);
    if (!d_net.p || !d_X.p || !d_Y.p || !d_bias.p) FAIL(103, "hipMalloc failed");
    if (hipMemcpy(d_net.p, net, net_bytes, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(d_X.p, X.data(), 4ull * B * n, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(d_bias.p, bias.data(), 4ull * m, hipMemcpyHostToDevice) != hipSuccess) FAIL(104, "hipMemcpy failed");
    hac_layer_t layers[2];
    std::memset(layers, 0, sizeof layers);
    layers[0].desc = &d0; layers[0].d_blob = d_net.p; layers[0].d_bias = static_cast<const float*>(d_bias.p); layers[0].activation = HAC_ACT_RELU;
    layers[1].desc = &d1; layers[1].d_blob = d_net.p;
    const size_t fw_bytes = hac_forward_workspace_bytes(layers, 2, B);
    DevBuf d_ws(fw_bytes);
    if (!d_ws.p) FAIL(105, "hipMalloc failed");
    rc = hac_forward(layers, 2, static_cast<const float*>(d_X.p), B, n, static_cast<float*>(d_Y.p), m2, d_ws.p, fw_bytes, stream);
    if (rc) FAIL(106, "forward: %s (hip %d)", hac_strerror(rc), hac_last_hip_error());
    if (hipStreamSynchronize(stream) != hipSuccess) FAIL(107, "stream failed");
    std::vector<float> Y((size_t)B * m2);
    if (hipMemcpy(Y.data(), d_Y.p, 4ull * B * m2, hipMemcpyDeviceToHost) != hipSuccess) FAIL(108, "copy back failed");
    for (int b = 0; b < B; ++b) {
        std::vector<double> a((size_t)m), abs_a((size_t)m);
        for (int j = 0; j < m; ++j) {
            double ref = 0.0, scale = 0.0;
            for (int i = 0; i < n; ++i) { const double t = (double)X[(size_t)b * n + i] * W[(size_t)i * m + j]; ref += t; scale += std::fabs(t); }
            ref += bias[(size_t)j];
            a[(size_t)j] = ref > 0 ? ref : 0.0;
            abs_a[(size_t)j] = 1e-5 * scale + 1.2e-7 * (std::fabs(ref) + std::fabs((double)bias[(size_t)j]));   // what layer 0 may be off by
        }
        for (int j = 0; j < m2; ++j) {
            double ref = 0.0, bound = 0.0;
            for (int i = 0; i < m; ++i) {
                const double w = W2[(size_t)i * m2 + j];
                ref += a[(size_t)i] * w;
                bound += abs_a[(size_t)i] * std::fabs(w) + 1e-5 * (a[(size_t)i] + abs_a[(size_t)i]) * std::fabs(w);
            }
            if (std::fabs((double)Y[(size_t)b * m2 + j] - ref) > bound + 1e-30) FAIL(109, "chain: row %d column %d off", b, j);
        }
    }
    hac_free(net);
    (void)hipStreamDestroy(stream);
    return 0;
}
