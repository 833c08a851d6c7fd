#include "laser_internal.h"
namespace laser {
bool gsta_tiled_supports(const GstaArgs&) { return false; }
laser_status gsta_tiled_launch(const GstaArgs&) { return LASER_ERR_UNSUPPORTED; }
}  // namespace laser
