// Host-side conversion of fp32 weight matrices into the streaming tile layout
// described at bild::TMat.  Runs once per model upload.
#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

#include "bild_internal.h"

namespace bild {

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    uint32_t r = ((u >> 16) & 1u) + 0x7FFFu;
    return (uint16_t)((u + r) >> 16);
}

size_t tiled_bytes(int n, int k, int dtype) {
    const int kt = dtype == BILD_DT_BF16 ? 32 : 16;
    return (size_t)((n + 15) / 16) * (size_t)(k / kt) * kTileBytes;
}

template <class F>
static void parallel_for(int n, F f) {
    int nthr = (int)std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
    nthr = std::min(nthr, std::max(1, n));
    if (nthr <= 1) {
        for (int i = 0; i < n; ++i) f(i);
        return;
    }
    std::vector<std::thread> th;
    for (int t = 0; t < nthr; ++t)
        th.emplace_back([=] {
            for (int i = t; i < n; i += nthr) f(i);
        });
    for (auto& x : th) x.join();
}

void tile_matrix(const float* src, bool src_is_k_by_n, int n, int k, int dtype, void* dst) {
    const int kt = dtype == BILD_DT_BF16 ? 32 : 16;
    const int per_lane = kt / 4;  // inputs held by one lane
    const int tn = (n + 15) / 16, tk = k / kt;
    parallel_for(tn, [=](int bn) {
        for (int bk = 0; bk < tk; ++bk) {
            char* tile = (char*)dst + ((size_t)bn * tk + bk) * kTileBytes;
            for (int lane = 0; lane < 64; ++lane) {
                const int f = bn * 16 + (lane & 15);
                const int k0 = bk * kt + (lane >> 4) * per_lane;
                for (int j = 0; j < per_lane; ++j) {
                    float v = 0.f;
                    if (f < n) v = src_is_k_by_n ? src[(size_t)(k0 + j) * n + f] : src[(size_t)f * k + k0 + j];
                    if (dtype == BILD_DT_BF16)
                        ((uint16_t*)(tile + lane * 16))[j] = f32_to_bf16_rne(v);
                    else
                        ((float*)(tile + lane * 16))[j] = v;
                }
            }
        }
    });
}

void tile_concat(const float* const* srcs, const int* ns, int count, int k, int dtype, void* dst) {
    size_t off = 0;
    for (int i = 0; i < count; ++i) {
        tile_matrix(srcs[i], true, ns[i], k, dtype, (char*)dst + off);
        off += tiled_bytes(ns[i], k, dtype);
    }
}

void tile_gated_pair(const float* gate, const float* up, int n, int k, int dtype, void* dst) {
    // n is a multiple of 16: feature tile j of the gate goes to tile 2j, of the up branch to 2j+1
    const int kt = dtype == BILD_DT_BF16 ? 32 : 16;
    const int tn = n / 16, tk = k / kt;
    const size_t strip = (size_t)tk * kTileBytes;
    std::vector<char> tmp_g(tiled_bytes(n, k, dtype)), tmp_u(tiled_bytes(n, k, dtype));
    tile_matrix(gate, true, n, k, dtype, tmp_g.data());
    tile_matrix(up, true, n, k, dtype, tmp_u.data());
    for (int j = 0; j < tn; ++j) {
        std::memcpy((char*)dst + (size_t)(2 * j) * strip, tmp_g.data() + (size_t)j * strip, strip);
        std::memcpy((char*)dst + (size_t)(2 * j + 1) * strip, tmp_u.data() + (size_t)j * strip, strip);
    }
}

}  // namespace bild
