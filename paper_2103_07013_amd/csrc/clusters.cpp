// Cluster builder: triangles are ordered along a Morton curve through their centroids; clusters
// are seeded in that order and grown over the mesh's vertex adjacency into compact patches of at
// most 64 distinct vertices and 128 triangles.
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
// Candidate triangles kept per growing cluster.  Ordinary meshes stay far below it; the bound keeps
// the work per cluster fixed on meshes with vertices of enormous valence (triangles left out are
// simply picked up by a later cluster).
constexpr size_t kMaxCandidates = 512;

// The renderer tests 64 consecutive clusters as one block.  Median splits along the longest axis of
// the cluster centres, cut at multiples of 64, put clusters that are close in space into the same
// block (much tighter block boxes than runs of a space-filling curve give).
void split_blocks(std::vector<uint32_t>& order, size_t first, size_t last, const std::vector<float>& centre) {
    const size_t n = last - first;
    if (n <= 64) return;
    float lo[3] = {INFINITY, INFINITY, INFINITY}, hi[3] = {-INFINITY, -INFINITY, -INFINITY};
    for (size_t i = first; i < last; ++i)
        for (int a = 0; a < 3; ++a) {
            lo[a] = std::min(lo[a], centre[3 * (size_t)order[i] + a]);
            hi[a] = std::max(hi[a], centre[3 * (size_t)order[i] + a]);
        }
    int axis = 0;
    for (int a = 1; a < 3; ++a)
        if (hi[a] - lo[a] > hi[axis] - lo[axis]) axis = a;
    const size_t mid = first + ((n + 63) / 64 / 2) * 64;
    std::nth_element(order.begin() + first, order.begin() + mid, order.begin() + last, [&](uint32_t x, uint32_t y) {
        const float fx = centre[3 * (size_t)x + axis], fy = centre[3 * (size_t)y + axis];
        return fx < fy || (fx == fy && x < y);
    });
    split_blocks(order, first, mid, centre);
    split_blocks(order, mid, last, centre);
}

void order_for_blocks(ClusterSet& cs) {
    if (cs.count <= 64) return;
    std::vector<float> centre((size_t)cs.count * 3);
    for (uint32_t c = 0; c < cs.count; ++c)
        for (int a = 0; a < 3; ++a) centre[3 * (size_t)c + a] = 0.5f * (cs.bounds[6 * (size_t)c + a] + cs.bounds[6 * (size_t)c + 3 + a]);
    std::vector<uint32_t> order(cs.count);
    std::iota(order.begin(), order.end(), 0u);
    split_blocks(order, 0, cs.count, centre);
    ClusterSet out;
    out.count = cs.count;
    out.verts.resize(cs.verts.size());
    out.tris.resize(cs.tris.size());
    out.tri_id.resize(cs.tri_id.size());
    out.bounds.resize(cs.bounds.size());
    for (uint32_t c = 0; c < cs.count; ++c) {
        const size_t s = order[c];
        std::memcpy(&out.verts[(size_t)c * 192], &cs.verts[s * 192], 192 * sizeof(float));
        std::memcpy(&out.tris[(size_t)c * 128], &cs.tris[s * 128], 128 * sizeof(uint32_t));
        std::memcpy(&out.tri_id[(size_t)c * 128], &cs.tri_id[s * 128], 128 * sizeof(uint32_t));
        std::memcpy(&out.bounds[(size_t)c * 6], &cs.bounds[s * 6], 6 * sizeof(float));
    }
    cs = std::move(out);
}

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

    // ---- region growing
    // A cluster starts at the first unassigned triangle of the spatial order and grows by the
    // triangle that costs least: fewest vertices not yet in the cluster first, then the one whose
    // centroid is nearest the seed's in the maximum norm, which makes square axis-aligned patches
    // (compact clusters have small boxes and small screen footprints, which is what the renderer's
    // culling tests look at).  Candidates are the unassigned triangles that touch a vertex of the
    // cluster; where the mesh offers none (unconnected triangles) the next ones in spatial order
    // stand in.
    std::vector<uint32_t> vstart(V + 1, 0);
    for (size_t i = 0; i < (size_t)T * 3; ++i) ++vstart[indices[i] + 1];
    for (uint32_t v = 0; v < V; ++v) vstart[v + 1] += vstart[v];
    std::vector<uint32_t> vtris((size_t)T * 3);
    {
        std::vector<uint32_t> fill(vstart.begin(), vstart.end() - 1);
        for (uint32_t tt = 0; tt < T; ++tt)
            for (int k = 0; k < 3; ++k) vtris[fill[indices[3 * (size_t)tt + k]]++] = tt;
    }
    std::vector<uint32_t> vfirst(vstart.begin(), vstart.end() - 1);   // first entry of a vertex's list that may be free
    std::vector<uint32_t> stamp(V, 0xFFFFFFFFu);     // cluster that last used the vertex
    std::vector<uint8_t> local(V, 0);
    std::vector<uint8_t> taken(T, 0);                // by triangle
    std::vector<uint32_t> listed(T, 0xFFFFFFFFu);    // cluster whose candidate list holds the triangle
    std::vector<uint32_t> cand;
    out.verts.reserve((size_t)(T / 90 + 1) * 192);
    out.tris.reserve((size_t)(T / 90 + 1) * 128);
    out.tri_id.reserve((size_t)(T / 90 + 1) * 128);

    uint32_t head = 0;  // first position of the spatial order not yet assigned
    while (true) {
        while (head < T && taken[(uint32_t)keyed[head]]) ++head;
        if (head >= T) break;
        const uint32_t c = out.count++;
        size_t vbase = out.verts.size(), tbase = out.tris.size();
        out.verts.resize(vbase + 192, 0.0f);
        out.tris.resize(tbase + 128, 0u);
        out.tri_id.resize(tbase + 128, 0xFFFFFFFFu);
        uint32_t nv = 0, nt = 0;
        float bl[3] = {INFINITY, INFINITY, INFINITY}, bh[3] = {-INFINITY, -INFINITY, -INFINITY};
        cand.clear();

        auto fresh_of = [&](uint32_t tt) {
            const uint32_t* ix = indices + 3 * (size_t)tt;
            uint32_t d = stamp[ix[0]] != c ? 1u : 0u;
            if (ix[1] != ix[0] && stamp[ix[1]] != c) ++d;
            if (ix[2] != ix[0] && ix[2] != ix[1] && stamp[ix[2]] != c) ++d;
            return d;
        };
        float seed_c[3];
        auto growth_of = [&](uint32_t tt) {
            float g = 0.0f;
            for (int a = 0; a < 3; ++a) {
                float m = 0.0f;
                for (int k = 0; k < 3; ++k) m += vertices[3 * (size_t)indices[3 * (size_t)tt + k] + a];
                g = std::max(g, std::fabs(m * (1.0f / 3.0f) - seed_c[a]));
            }
            return g;
        };
        auto add = [&](uint32_t tt) {
            taken[tt] = 1;
            uint32_t li[3];
            for (int k = 0; k < 3; ++k) {
                const uint32_t vi = indices[3 * (size_t)tt + k];
                if (stamp[vi] != c) {
                    stamp[vi] = c;
                    local[vi] = (uint8_t)nv;
                    for (int a = 0; a < 3; ++a) {
                        const float f = vertices[3 * (size_t)vi + a];
                        out.verts[vbase + 64 * a + nv] = f;
                        bl[a] = std::min(bl[a], f);
                        bh[a] = std::max(bh[a], f);
                    }
                    ++nv;
                    // triangles once taken stay taken: skip the taken head of the vertex's list for good
                    uint32_t& from = vfirst[vi];
                    while (from < vstart[vi + 1] && taken[vtris[from]]) ++from;
                    for (uint32_t q = from; q < vstart[vi + 1] && cand.size() < kMaxCandidates; ++q) {
                        const uint32_t o = vtris[q];
                        if (!taken[o] && listed[o] != c) {
                            listed[o] = c;
                            cand.push_back(o);
                        }
                    }
                }
                li[k] = local[vi];
            }
            out.tris[tbase + nt] = li[0] | (li[1] << 8) | (li[2] << 16);
            out.tri_id[tbase + nt] = tt;
            ++nt;
        };

        for (int a = 0; a < 3; ++a) {
            float m = 0.0f;
            for (int k = 0; k < 3; ++k) m += vertices[3 * (size_t)indices[3 * (size_t)(uint32_t)keyed[head] + k] + a];
            seed_c[a] = m * (1.0f / 3.0f);
        }
        add((uint32_t)keyed[head]);     // the seed keeps the clusters in spatial order
        while (nt < kClusterTris) {
            uint32_t best = 0xFFFFFFFFu, best_new = 4;
            float best_grow = INFINITY;
            size_t keep = 0;
            for (size_t q = 0; q < cand.size(); ++q) {
                const uint32_t tt = cand[q];
                if (taken[tt]) continue;
                cand[keep++] = tt;          // drop assigned triangles from the list as we go
                const uint32_t fresh = fresh_of(tt);
                if (fresh > best_new) continue;
                const float grow = growth_of(tt);
                if (fresh < best_new || grow < best_grow) {
                    best_new = fresh;
                    best_grow = grow;
                    best = tt;
                }
            }
            cand.resize(keep);
            if (best == 0xFFFFFFFFu) {
                // nothing connected is left: look at the next triangles of the spatial order
                uint32_t seen = 0;
                for (uint32_t p = head; p < T && seen < kWindow; ++p) {
                    const uint32_t tt = (uint32_t)keyed[p];
                    if (taken[tt]) continue;
                    ++seen;
                    const uint32_t fresh = fresh_of(tt);
                    if (fresh < best_new) {
                        best_new = fresh;
                        best = tt;
                        if (fresh == 0) break;
                    }
                }
            }
            if (best == 0xFFFFFFFFu || nv + best_new > kClusterVerts) break;
            add(best);
        }
        for (uint32_t l = nv; l < kClusterVerts; ++l)
            for (int a = 0; a < 3; ++a) out.verts[vbase + 64 * a + l] = out.verts[vbase + 64 * a];
        out.tris[tbase] |= nt << 24;
        for (int a = 0; a < 3; ++a) out.bounds.push_back(bl[a]);
        for (int a = 0; a < 3; ++a) out.bounds.push_back(bh[a]);
    }
    order_for_blocks(out);
    return out;
}

}  // namespace bps
