#include "st_internal.h"
namespace st {
hipError_t launch_fwd_bf16(const FwdArgs&, hipStream_t) { return hipErrorNotSupported; }
}
