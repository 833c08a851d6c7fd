#include "laser_internal.h"
namespace laser {
bool sta_stream_supports(const StaArgs&) { return false; }
laser_status sta_stream_launch(const StaArgs&) { return LASER_ERR_UNSUPPORTED; }
}  // namespace laser
