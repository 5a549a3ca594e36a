// Host-side re-packing of an indexed triangle mesh into fixed-size clusters.
//
// A cluster holds at most 64 distinct vertices and 128 triangles, so one 64-lane wavefront
// transforms each vertex of a cluster once (one lane per vertex) and then handles two
// triangles per lane.  This is part of scene upload (paper Sec. 3.2 "Scene asset sharing"),
// off the per-frame path.
#pragma once
#include <cstdint>
#include <vector>

namespace bps {

constexpr uint32_t kClusterVerts = 64;
constexpr uint32_t kClusterTris = 128;

struct ClusterSet {
    uint32_t count = 0;
    // per cluster: x[64], y[64], z[64]; unused lanes repeat the cluster's first vertex
    std::vector<float> verts;
    // per cluster: 128 words, local indices i0 | i1 << 8 | i2 << 16; unused slots are 0 (a
    // degenerate triangle); bits 24..31 of word 0 hold the number of used slots
    std::vector<uint32_t> tris;
    // per cluster: 128 words, row of the triangle in the caller's index array (0xFFFFFFFF unused)
    std::vector<uint32_t> tri_id;
    // per cluster: axis-aligned bounds, min xyz then max xyz
    std::vector<float> bounds;
};

// vertices [V][3], indices [T][3]; every index must already be < V.
ClusterSet build_clusters(const float* vertices, uint32_t V, const uint32_t* indices, uint32_t T);

}  // namespace bps
