// placeholder until the backward kernels land
#include "attn_common.h"
namespace attn {
int launch_bwd(const KArgs&, int, int, bool, bool, bool, hipStream_t) { return (int)hipErrorNotSupported; }
}
