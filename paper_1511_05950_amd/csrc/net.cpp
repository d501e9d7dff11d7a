// placeholder
#include "ctx.hpp"
namespace sasgd {
struct Net {};
int net_create(const sasgd_config&, Net**, int64_t*, size_t*, std::string& err) { err = "network path not built"; return SASGD_EINVAL; }
void net_destroy(Net*) {}
size_t net_workspace_bytes(const Net*) { return 0; }
void net_set_workspace(Net*, int, void*) {}
hipError_t net_prepare_version(Net*, const void*, void*, hipStream_t) { return hipSuccess; }
hipError_t net_calc_gradient(Net*, const int*, const LearnerBind*, int, float*, hipStream_t) { return hipErrorNotSupported; }
}
