// Host planner: turns the strided pieces of a map into kernel launches.
#pragma once

#include <vector>

#include "amap_device.hpp"
#include "amap_map.hpp"

namespace amap_detail {

struct Plan {
    bool fits32 = true;                         // every tensor has < 2^31 elements
    bool strided_ok = false;                    // launches[] is valid
    bool windowed = false;                      // pieces carry 64-bit window origins (a tensor exceeds 32-bit offsets)
    std::vector<amap_dev::LaunchArgs> launches; // DevPiece::src holds (source id + 1) until launch
    std::vector<uint32_t> grid;                 // workgroups per launch
    std::vector<uint32_t> lds_bytes;            // dynamic LDS per launch
    bool program_ok = false;                    // prog is valid
    amap_dev::Program prog;
    int n_prog_src = 0;
    int main_kernel = AMAP_K_PROGRAM;           // family of the largest piece
    int min_vec_bytes = 0;
};

// family: -1 = choose per piece; otherwise an amap_kernel_id to force
// (AMAP_K_ELEMENT, AMAP_K_ROWS, AMAP_K_TILE, AMAP_K_WAVE).
// Returns false if some piece cannot run in the forced family.
bool plan_strided(const amap &m, int family, Plan &out);

// Flatten the operator program; false if it does not fit the argument block.
bool plan_program(const amap &m, Plan &out);

// Build and attach the default plan (called when a map is finalised).
void attach_plan(amap &m);

// Remember the text behind an AMAP_E_HIP for amap_last_error() (per thread).
void set_last_error(const char *what, const char *detail = nullptr);

inline const Plan *plan_of(const amap &m) { return static_cast<const Plan *>(m.plan.get()); }

}  // namespace amap_detail
