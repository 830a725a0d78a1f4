// placeholder until the network executor lands
#include "net.h"
struct Net { int dummy; };
Net *net_create(const parle_config &, const Arch &, const std::vector<Segment> &, int64_t, std::string &err) { return new Net{0}; }
void net_destroy(Net *net) { delete net; }
int64_t net_workspace_bytes(const Net *) { return 0; }
int64_t net_bn_floats_per_replica(const Net *) { return 0; }
hipError_t net_train_step(Net *, hipStream_t, const float *, const void *, float *, float *, void *, const float *, const int32_t *, float *) { return hipErrorNotSupported; }
hipError_t net_eval(Net *, hipStream_t, const float *, const float *, void *, const float *, const int32_t *, int, float *, int32_t *) { return hipErrorNotSupported; }
hipError_t net_average_bn(Net *, hipStream_t, const float *, float *) { return hipErrorNotSupported; }
hipError_t net_init_bn(Net *, hipStream_t, float *) { return hipErrorNotSupported; }
