// HIP source generation for "uvw" problems (the paper's sub-kernel C: dense weight tile).
#include <stdexcept>

#include "plan.hpp"

namespace cgtp {

int64_t uvw_tile_samples(const Plan&) { return 32; }

void emit_uvw_forward(const Plan&, Kernel&) { throw std::runtime_error("uvw forward is not implemented yet"); }

}  // namespace cgtp
