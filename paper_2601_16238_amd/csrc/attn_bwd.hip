#include "attn_device.hpp"
#include "attn_launch.hpp"
namespace attn {
int launch_bwd(const BwdArgs &, int, bool, hipStream_t) { return -1; }
}
