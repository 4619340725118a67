// Internal interface of the host-side tuner (shared by tune.cpp and the launch code).
#ifndef IOLB_TUNE_H
#define IOLB_TUNE_H

#include "iolbconv.h"

#include <array>
#include <cstdint>
#include <vector>

namespace iolb {

struct Candidate {
    iolb_tile_config cfg;
    std::array<int64_t, 10> key;     // this build's order (modelled time first): lexicographic, smaller is better
    std::array<int64_t, 10> volume;   // the paper's order: reading volume of the dataflow, then distance from the
                                     // optimality condition x y = R z, then the fuller block
};

// Output tile extent m of a Winograd algo id, 0 for anything else.
int winograd_m(int algo);
// Checks a layer description and computes its output extents.
int validate_shape(const iolb_shape& s, int* P, int* Q);
// All feasible tiles, best first.
int enumerate(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, bool use_box, std::vector<Candidate>* out);
// Every plain-FMA tile of a direct layer (the fallback path), whole domain, best first.
int enumerate_fma(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, std::vector<Candidate>* out);
// The best tile (box first, whole domain if the box is empty).
int tune(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, iolb_tile_config* cfg);
// The tile of least reading volume inside the optimality box (whole domain if the box is empty).
int tune_by_volume(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, iolb_tile_config* cfg);
int bounds(const iolb_shape& s, int64_t Sf, iolb_bounds_out* o);

}  // namespace iolb

#endif
