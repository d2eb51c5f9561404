// placeholder until the MFMA kernel lands
#include "lasad_internal.h"
namespace lasad {
hipError_t launch_forward_mfma(const ForwardArgs &a, hipStream_t s) { return launch_forward_generic(a, s); }
}
