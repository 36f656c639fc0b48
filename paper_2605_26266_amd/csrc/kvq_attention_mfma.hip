// placeholder until the matrix-core kernel lands
#include "kvq_internal.h"
namespace kvq {
hipError_t launch_attention_mfma(const AttentionArgs &, hipStream_t) { return hipErrorNotSupported; }
}
