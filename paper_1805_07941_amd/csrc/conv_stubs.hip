#include "dfq_host.hpp"
namespace dfq {
bool conv_depthwise_supports(const ConvArgs &) { return false; }
hipError_t launch_conv_depthwise(const ConvArgs &, hipStream_t) { return hipErrorNotSupported; }
bool conv_smallc_supports(const ConvArgs &) { return false; }
hipError_t launch_conv_smallc(const ConvArgs &, hipStream_t) { return hipErrorNotSupported; }
}
