// Host-side robustness driver, meant to be built with -fsanitize=address,undefined:
// encodes a few small matrices in every format, checks the round trip, then damages the blobs
// at random (byte flips, truncation, header pokes) and runs the validator and the decoder on
// them.  Whatever they answer, they must not read or write out of bounds.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/hac.h"

static std::vector<float> make_matrix(std::mt19937& rng, int n, int m, double density, int k)
{
    std::vector<float> vals(k);
    for (int i = 0; i < k; ++i) vals[i] = (float)(i + 1) * 0.25f - (float)(k / 2);
    for (auto& v : vals) if (v == 0.0f) v = 0.125f;
    std::vector<float> W((size_t)n * m, 0.0f);
    std::uniform_real_distribution<double> u(0.0, 1.0);
    for (auto& w : W) if (u(rng) < density) w = vals[rng() % k];
    return W;
}

static int exercise(const void* blob, size_t bytes, int n, int m, const std::vector<float>* expect)
{
    hac_desc_t d;
    if (hac_describe(blob, bytes, &d) != HAC_OK) return 0;
    const int ok = hac_validate(blob, bytes, 1);
    hac_validate(blob, bytes, 0);
    hac_stats_t st;
    hac_stats(blob, bytes, &st);
    if (ok != HAC_OK) return 0;
    if (d.n != (uint64_t)n || d.m != (uint64_t)m) return 0;       // a damaged header that still validates: do not size buffers from it
    std::vector<float> W((size_t)n * m, -1.0f);
    std::vector<int32_t> sym((size_t)n * m + 1), row((size_t)n * m + 1), col((size_t)n * m + 1);
    const bool csc = d.format == HAC_FORMAT_SHAC;
    if (csc && d.nnz > (uint64_t)n * m) return 0;
    const int rc = hac_decode_host(blob, bytes, W.data(), sym.data(), csc ? row.data() : nullptr, csc ? col.data() : nullptr);
    if (expect && (rc != HAC_OK || std::memcmp(W.data(), expect->data(), W.size() * 4) != 0)) {
        std::fprintf(stderr, "round trip failed (format %u)\n", d.format);
        return 1;
    }
    return 0;
}

// the same for a network blob of two layers (n x m, then m x n2)
static int exercise_net(const void* blob, size_t bytes, const int64_t* ns, const int64_t* ms,
                        const std::vector<float>* const* expect)
{
    hac_net_t net;
    if (hac_net_describe(blob, bytes, &net) != HAC_OK) return 0;
    const int ok = hac_net_validate(blob, bytes, 1);
    hac_net_validate(blob, bytes, 0);
    hac_net_stats_t st;
    hac_net_stats(blob, bytes, &st);
    if (ok != HAC_OK || net.n_layers != 2) return 0;
    for (uint32_t l = 0; l < 2; ++l) {
        hac_desc_t d;
        if (hac_net_layer(blob, bytes, l, &d) != HAC_OK) return 0;
        if (d.n != (uint64_t)ns[l] || d.m != (uint64_t)ms[l] || d.nnz > d.n * d.m) return 0;
        const size_t nm = (size_t)(ns[l] * ms[l]);
        std::vector<float> W(nm, -1.0f);
        std::vector<int32_t> sym(nm + 1), row(nm + 1), col(nm + 1);
        const bool csc = d.format == HAC_FORMAT_SHAC;
        const int rc = hac_net_decode_host(blob, bytes, l, W.data(), sym.data(), csc ? row.data() : nullptr,
                                           csc ? col.data() : nullptr);
        if (expect && (rc != HAC_OK || std::memcmp(W.data(), expect[l]->data(), nm * 4) != 0)) {
            std::fprintf(stderr, "network round trip failed (layer %u, format %u)\n", l, d.format);
            return 1;
        }
    }
    return 0;
}

static void fuzz_networks(std::mt19937& rng, int& failures, long& cases)
{
    const int shapes[][3] = { {1, 1, 1}, {9, 6, 4}, {40, 33, 7}, {120, 10, 50} };
    for (const auto& sh : shapes)
        for (double density : { 0.0, 0.1, 0.7 })
            for (int k : { 1, 5, 120 })
                for (int f = 0; f < 9; ++f) {
                    const int64_t ns[2] = { sh[0], sh[1] }, ms[2] = { sh[1], sh[2] };
                    std::vector<float> W0 = make_matrix(rng, sh[0], sh[1], density, k);
                    std::vector<float> W1 = make_matrix(rng, sh[1], sh[2], f % 2 ? density : 1.0 - density, k + 2);
                    const std::vector<float>* expect[2] = { &W0, &W1 };
                    const float* Ws[2] = { W0.data(), W1.data() };
                    // f = 0..5: HAC / sHAC pairs (4, 5 with Rice-coded gaps); 6..8: an index map beside them
                    uint32_t fm[2] = { (uint32_t)(f & 1 ? HAC_FORMAT_SHAC : HAC_FORMAT_HAC),
                                       (uint32_t)(f & 2 ? HAC_FORMAT_SHAC : HAC_FORMAT_HAC) };
                    if (f == 6) fm[0] = HAC_FORMAT_IM;
                    if (f == 7) fm[1] = HAC_FORMAT_IM;
                    if (f == 8) fm[0] = fm[1] = HAC_FORMAT_IM;
                    hac_opts_t o; std::memset(&o, 0, sizeof o);
                    o.ri_coding = (f == 4 || f == 5) ? HAC_RI_RICE : HAC_RI_FIELDS;
                    o.chunk_nnz = (uint32_t)(rng() % 3 == 0 ? 1 + rng() % 9 : 0);
                    void* blob = nullptr; size_t bytes = 0;
                    const int rc = hac_net_encode(2, fm, Ws, ns, ms, ms, &o, &blob, &bytes);
                    if (rc != HAC_OK) { std::fprintf(stderr, "network encode failed: %d\n", rc); ++failures; continue; }
                    failures += exercise_net(blob, bytes, ns, ms, expect);
                    ++cases;
                    std::vector<uint8_t> copy((const uint8_t*)blob, (const uint8_t*)blob + bytes);
                    for (int t = 0; t < 40; ++t) {
                        std::vector<uint8_t> bad = copy;
                        const int kind = (int)(rng() % 4);
                        if (kind == 0) bad[rng() % bad.size()] ^= (uint8_t)(1u << (rng() % 8));
                        else if (kind == 1) bad[rng() % 768] = (uint8_t)rng();                       // the three headers
                        else if (kind == 2) { for (int q = 0; q < 8; ++q) bad[rng() % bad.size()] = (uint8_t)rng(); }
                        else bad.resize(rng() % bad.size());
                        uint8_t* heap = (uint8_t*)std::malloc(bad.size() ? bad.size() : 1);
                        std::memcpy(heap, bad.data(), bad.size());
                        failures += exercise_net(heap, bad.size(), ns, ms, nullptr);
                        failures += exercise(heap, bad.size(), sh[0], sh[1], nullptr);               // and as if it were a layer blob
                        std::free(heap);
                        ++cases;
                    }
                    hac_free(blob);
                }
}

int main()
{
    std::mt19937 rng(12345);
    int failures = 0;
    long cases = 0;
    const int shapes[][2] = { {1, 1}, {7, 5}, {64, 3}, {33, 40}, {300, 17} };
    for (const auto& sh : shapes) {
        for (double density : { 0.0, 0.05, 0.5, 1.0 }) {
            for (int k : { 1, 3, 40, 300 }) {
                const int n = sh[0], m = sh[1];
                std::vector<float> W = make_matrix(rng, n, m, density, k);
                for (int f = 0; f < 4; ++f) {
                    void* blob = nullptr; size_t bytes = 0;
                    hac_opts_t o; std::memset(&o, 0, sizeof o);
                    o.chunk_nnz = (uint32_t)(rng() % 3 == 0 ? 1 + rng() % 9 : 0);
                    // half of the HAC and sHAC blobs carry the row index (rows per entry: automatic,
                    // a small multiple of 4, or the whole column)
                    if (f < 2 && rng() % 2 == 0) {
                        const uint32_t pick = (uint32_t)(rng() % 3);
                        o.chunk_rows = pick == 0 ? HAC_CHUNK_ROWS_AUTO : pick == 1 ? (uint32_t)n : 4u * (1u + (uint32_t)(rng() % 4));
                        if (o.chunk_rows != HAC_CHUNK_ROWS_AUTO && o.chunk_rows > (uint32_t)n) o.chunk_rows = (uint32_t)n;
                    }
                    int rc;
                    if (f == 0) rc = hac_encode(W.data(), n, m, m, &o, &blob, &bytes);
                    else if (f == 1) rc = shac_encode(W.data(), n, m, m, &o, &blob, &bytes);
                    else if (f == 2) { o.ri_coding = HAC_RI_RICE; rc = shac_encode(W.data(), n, m, m, &o, &blob, &bytes); }
                    else rc = im_encode(W.data(), n, m, m, nullptr, &blob, &bytes);
                    if (rc != HAC_OK) { std::fprintf(stderr, "encode %d failed: %d\n", f, rc); ++failures; continue; }
                    failures += exercise(blob, bytes, n, m, &W);
                    ++cases;
                    std::vector<uint8_t> copy((const uint8_t*)blob, (const uint8_t*)blob + bytes);
                    for (int t = 0; t < 60; ++t) {
                        std::vector<uint8_t> bad = copy;
                        const int kind = (int)(rng() % 4);
                        if (kind == 0) bad[rng() % bad.size()] ^= (uint8_t)(1u << (rng() % 8));
                        else if (kind == 1) bad[rng() % 256] = (uint8_t)rng();                       // header
                        else if (kind == 2) { for (int q = 0; q < 8; ++q) bad[rng() % bad.size()] = (uint8_t)rng(); }
                        else bad.resize(rng() % bad.size());                                          // truncated
                        // give the library an exactly-sized heap copy so that any over-read is caught
                        uint8_t* heap = (uint8_t*)std::malloc(bad.size() ? bad.size() : 1);
                        std::memcpy(heap, bad.data(), bad.size());
                        failures += exercise(heap, bad.size(), n, m, nullptr);
                        std::free(heap);
                        ++cases;
                    }
                    hac_free(blob);
                }
            }
        }
    }
    fuzz_networks(rng, failures, cases);
    std::printf("host fuzz: %ld cases, %d failures\n", cases, failures);
    return failures ? 1 : 0;
}
