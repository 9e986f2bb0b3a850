// Configuration-space encoder: the four parameter types of Sec. 3 with their adjacency
// graphs, the Cartesian product of Eq. 1, and the q-random walk of Sec. 4.3.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "common.hpp"

namespace opevo {

struct Param {
    int type = OPEVO_FACTOR;
    int nu = 0;
    int64_t C = 0;
    int n_values = 0;
    std::vector<double> values;
    std::string name;
    int width = 0;    // int32 slots in the flat encoding
    int offset = 0;   // first slot
    int64_t n_verts = 0;
    std::vector<int32_t> verts;  // n_verts * width, canonical order

    // Position of vertex v in the canonical order, -1 if v is not a vertex.
    int64_t index_of(const int32_t *v) const;
    const int32_t *vertex(int64_t i) const { return verts.data() + i * width; }
    // Appends S(v) to out (flattened vertices) in the canonical order; returns |S(v)|.
    int neighbors(const int32_t *v, std::vector<int32_t> &out) const;
    // One q-random walk in place.
    void walk(double q, Rng &rng, int32_t *v, std::vector<int32_t> &scratch) const;
};

}  // namespace opevo

struct opevo_space {
    std::vector<opevo::Param> params;
    int width = 0;

    bool is_legal(const int32_t *cfg) const;
    double size() const;
    bool rankable() const;                 // fewer than 2^62 members
    int64_t rank(const int32_t *cfg) const;  // -1 if illegal
    void unrank(int64_t r, int32_t *cfg) const;
    void random(opevo::Rng &rng, int32_t *cfg) const;
    void mutate(double q, opevo::Rng &rng, int32_t *cfg) const;
    // Control mutation that ignores the graphs: per parameter, with probability q a uniformly random vertex.
    void mutate_uniform(double q, opevo::Rng &rng, int32_t *cfg) const;
};
