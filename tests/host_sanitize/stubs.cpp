// Device half of the library replaced by refusals, so that the host half - inspector, code
// generator, serialisation, boundary - links without a HIP runtime and can run under the host
// sanitizers.  Test infrastructure only.
#include "../../paper_2008_11849_amd/csrc/plan.h"

namespace sparsert {

int upload_plan(const HostPlan &, DevicePlan &, std::string &err) { err = "host build: no device"; return SPARSERT_EHIP; }
void free_device_plan(DevicePlan &d) { d = DevicePlan(); }
bool on_plan_device(const DevicePlan &) { return false; }
int launch_rows(const HostPlan &, const DevicePlan &, const void *, void *, void *, std::string &err) { err = "host build: no device"; return SPARSERT_EHIP; }
int launch_spec(const HostPlan &, const DevicePlan &, const void *, void *, void *, std::string &err) { err = "host build: no device"; return SPARSERT_EHIP; }

int compare_with_own_partials(const HostPlan &, const void *, const void *, uint32_t *, void *, std::string &err) { err = "host build: no device"; return SPARSERT_EHIP; }

int launch_compare(const HostPlan &, const void *, const void *, uint32_t *, uint32_t *, void *, std::string &err) { err = "host build: no device"; return SPARSERT_EHIP; }
int static_compare_scratch(uint32_t **, std::string &err) { err = "host build: no device"; return SPARSERT_EHIP; }
int64_t static_compare_max_elements() { return 0; }

}  // namespace sparsert
