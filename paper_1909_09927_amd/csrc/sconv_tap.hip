// placeholder: element-stationary 3x3 kernel (not yet enabled)
#include "sconv_internal.h"
namespace sconv {
bool tap_supported(const Problem&, bool) { return false; }
int launch_tap(const Problem&, bool, const float*, const float*, float*, hipStream_t) { return SCONV_EUNSUPPORTED; }
}
