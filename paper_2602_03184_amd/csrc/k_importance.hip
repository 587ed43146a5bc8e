// placeholder until the Alg. 1 kernel lands: refuse loudly
#include "dsk_internal.hpp"
namespace dsk {
hipError_t launch_importance(const dsk_compress_args&, const CompressWs&, hipStream_t) { return hipErrorNotSupported; }
}
