// Cluster builder: order triangles along a Morton curve through their centroids so that
// neighbours in the list are neighbours in space, then cut the list greedily whenever the
// next triangle would not fit (more than 64 distinct vertices or more than 128 triangles).
// A short look-ahead window prefers triangles that reuse vertices already in the cluster.
#include "clusters.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

namespace bps {
namespace {

inline uint32_t spread10(uint32_t v) {  // 10 bits -> every third bit
    v &= 0x3FFu;
    v = (v | (v << 16)) & 0x030000FFu;
    v = (v | (v << 8)) & 0x0300F00Fu;
    v = (v | (v << 4)) & 0x030C30C3u;
    v = (v | (v << 2)) & 0x09249249u;
    return v;
}

constexpr uint32_t kWindow = 192;  // look-ahead, in triangles

}  // namespace

ClusterSet build_clusters(const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T) {
    ClusterSet out;
    if (T == 0 || V == 0) return out;

    // ---- spatial order
    float lo[3] = {INFINITY, INFINITY, INFINITY}, hi[3] = {-INFINITY, -INFINITY, -INFINITY};
    for (uint32_t v = 0; v < V; ++v)
        for (int a = 0; a < 3; ++a) {
            lo[a] = std::min(lo[a], vertices[3 * (size_t)v + a]);
            hi[a] = std::max(hi[a], vertices[3 * (size_t)v + a]);
        }
    float ext = std::max({hi[0] - lo[0], hi[1] - lo[1], hi[2] - lo[2], 1e-20f});
    float scale = 1023.0f / ext;
    std::vector<uint64_t> keyed(T);
    for (uint32_t t = 0; t < T; ++t) {
        uint32_t code = 0;
        for (int a = 0; a < 3; ++a) {
            float c = (vertices[3 * (size_t)indices[3 * (size_t)t + 0] + a] + vertices[3 * (size_t)indices[3 * (size_t)t + 1] + a] +
                       vertices[3 * (size_t)indices[3 * (size_t)t + 2] + a]) * (1.0f / 3.0f);
            uint32_t q = (uint32_t)std::min(1023.0f, std::max(0.0f, (c - lo[a]) * scale));
            code |= spread10(q) << a;
        }
        keyed[t] = ((uint64_t)code << 32) | t;
    }
    std::sort(keyed.begin(), keyed.end());

    // ---- greedy cut with look-ahead
    std::vector<uint32_t> stamp(V, 0xFFFFFFFFu);  // cluster that last used the vertex
    std::vector<uint8_t> local(V, 0);
    std::vector<uint8_t> taken(T, 0);             // position in `keyed` already assigned
    out.verts.reserve((size_t)(T / 90 + 1) * 192);
    out.tris.reserve((size_t)(T / 90 + 1) * 128);
    out.tri_id.reserve((size_t)(T / 90 + 1) * 128);

    uint32_t head = 0;  // first position not yet assigned
    while (head < T) {
        uint32_t c = out.count++;
        size_t vbase = out.verts.size(), tbase = out.tris.size();
        out.verts.resize(vbase + 192, 0.0f);
        out.tris.resize(tbase + 128, 0u);
        out.tri_id.resize(tbase + 128, 0xFFFFFFFFu);
        uint32_t nv = 0, nt = 0;
        float bl[3] = {INFINITY, INFINITY, INFINITY}, bh[3] = {-INFINITY, -INFINITY, -INFINITY};
        while (nt < kClusterTris) {
            while (head < T && taken[head]) ++head;
            if (head >= T) break;
            // pick, among the next kWindow unassigned triangles, the one adding fewest vertices
            uint32_t best = 0xFFFFFFFFu, best_new = 4, seen = 0;
            for (uint32_t p = head; p < T && seen < kWindow; ++p) {
                if (taken[p]) continue;
                ++seen;
                uint32_t t = (uint32_t)keyed[p];
                uint32_t fresh = 0;
                for (int k = 0; k < 3; ++k) fresh += stamp[indices[3 * (size_t)t + k]] != c;
                // repeated index inside one triangle counts once
                const uint32_t* ix = indices + 3 * (size_t)t;
                if (fresh > 1 && (ix[0] == ix[1] || ix[1] == ix[2] || ix[0] == ix[2])) {
                    uint32_t d = 0;
                    if (stamp[ix[0]] != c) ++d;
                    if (ix[1] != ix[0] && stamp[ix[1]] != c) ++d;
                    if (ix[2] != ix[0] && ix[2] != ix[1] && stamp[ix[2]] != c) ++d;
                    fresh = d;
                }
                if (fresh < best_new) {
                    best_new = fresh;
                    best = p;
                    if (fresh == 0) break;
                }
                // the head triangle is taken first when the cluster is empty, to keep spatial order
                if (nt == 0) break;
            }
            if (best == 0xFFFFFFFFu || nv + best_new > kClusterVerts) break;
            uint32_t t = (uint32_t)keyed[best];
            taken[best] = 1;
            uint32_t li[3];
            for (int k = 0; k < 3; ++k) {
                uint32_t vi = indices[3 * (size_t)t + k];
                if (stamp[vi] != c) {
                    stamp[vi] = c;
                    local[vi] = (uint8_t)nv;
                    for (int a = 0; a < 3; ++a) {
                        float f = vertices[3 * (size_t)vi + a];
                        out.verts[vbase + 64 * a + nv] = f;
                        bl[a] = std::min(bl[a], f);
                        bh[a] = std::max(bh[a], f);
                    }
                    ++nv;
                }
                li[k] = local[vi];
            }
            out.tris[tbase + nt] = li[0] | (li[1] << 8) | (li[2] << 16);
            out.tri_id[tbase + nt] = t;
            ++nt;
        }
        for (uint32_t l = nv; l < kClusterVerts; ++l)
            for (int a = 0; a < 3; ++a) out.verts[vbase + 64 * a + l] = out.verts[vbase + 64 * a];
        out.tris[tbase] |= nt << 24;
        for (int a = 0; a < 3; ++a) out.bounds.push_back(bl[a]);
        for (int a = 0; a < 3; ++a) out.bounds.push_back(bh[a]);
    }
    return out;
}

}  // namespace bps
