// placeholder until the graph walk lands
#include "host_common.hpp"
namespace gensor {
gensor_status construct_internal(const gensor_problem* p, const gensor_hw*, const gensor_construct_opts*, uint64_t seed, bool vec_ok, gensor_schedule* out) {
  GemmView v; gensor_status st = gemm_view(p, &v); if (st != GENSOR_OK) return st;
  for (int i = 0; i < g_num_instances; ++i) if (instance_serves(g_instances[i], v) && (vec_ok || !g_instances[i].vec) && !g_instances[i].direct) { schedule_from_instance(g_instances[i], out); out->seed = seed; return GENSOR_OK; }
  return GENSOR_ERR_NO_SCHEDULE;
}
}
extern "C" gensor_status gensor_construct(const gensor_problem* p, const gensor_hw* hw, const gensor_construct_opts* o, uint64_t seed, gensor_schedule* out) { return gensor::construct_internal(p, hw, o, seed, true, out); }
extern "C" const gensor_hw* gensor_hw_mi355x(void) { static gensor_hw h = {}; return &h; }
extern "C" gensor_status gensor_construct_trace(const gensor_problem*, const gensor_hw*, const gensor_construct_opts*, uint64_t, int32_t, int32_t*, int32_t*, int32_t*, int32_t*) { return GENSOR_ERR_UNSUPPORTED; }
extern "C" double gensor_predict_us(const gensor_schedule*, const gensor_problem*, const gensor_hw*) { return -1; }
