// Picks, by element format, one of the three builds of quantize_pack.hip.
#include "daf_internal.h"

#define DAF_DECLARE(dt)                                                                                              \
  hipError_t daf_launch_quantize_pack_batch_dt##dt(const daf_quantize_item_t*, int32_t, hipStream_t);               \
  hipError_t daf_launch_group_minmax_dt##dt(const daf_plan_t*, const void*, float*, float*, hipStream_t);            \
  hipError_t daf_launch_quantize_pack_dt##dt(const daf_plan_t*, const void*, uint64_t, uint32_t*, float*, float*,    \
                                             float*, void*, void*, hipStream_t);
DAF_DECLARE(0)
DAF_DECLARE(1)
DAF_DECLARE(2)
#undef DAF_DECLARE
int daf_quantize_route_dt0(const daf_plan_t*);
int daf_quantize_route_dt1(const daf_plan_t*);
int daf_quantize_route_dt2(const daf_plan_t*);

int daf_quantize_route(const daf_plan_t* plan, int dtype) {
  switch (dtype) {
    case 0: return daf_quantize_route_dt0(plan);
    case 1: return daf_quantize_route_dt1(plan);
    case 2: return daf_quantize_route_dt2(plan);
    default: return -1;
  }
}

hipError_t daf_launch_quantize_pack_batch(const daf_quantize_item_t* items, int32_t n_items, int dtype,
                                          hipStream_t stream) {
  switch (dtype) {
    case 0: return daf_launch_quantize_pack_batch_dt0(items, n_items, stream);
    case 1: return daf_launch_quantize_pack_batch_dt1(items, n_items, stream);
    case 2: return daf_launch_quantize_pack_batch_dt2(items, n_items, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t daf_launch_group_minmax(const daf_plan_t* plan, const void* x, int dtype, float* out_min, float* out_max,
                                   hipStream_t stream) {
  switch (dtype) {
    case 0: return daf_launch_group_minmax_dt0(plan, x, out_min, out_max, stream);
    case 1: return daf_launch_group_minmax_dt1(plan, x, out_min, out_max, stream);
    case 2: return daf_launch_group_minmax_dt2(plan, x, out_min, out_max, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t daf_launch_quantize_pack(const daf_plan_t* plan, const void* x, int dtype, uint64_t seed,
                                    uint32_t* out_words, float* out_min, float* out_scale, float* out_metrics,
                                    void* out_relu_y, void* big_scratch, hipStream_t stream) {
  switch (dtype) {
    case 0: return daf_launch_quantize_pack_dt0(plan, x, seed, out_words, out_min, out_scale, out_metrics, out_relu_y, big_scratch, stream);
    case 1: return daf_launch_quantize_pack_dt1(plan, x, seed, out_words, out_min, out_scale, out_metrics, out_relu_y, big_scratch, stream);
    case 2: return daf_launch_quantize_pack_dt2(plan, x, seed, out_words, out_min, out_scale, out_metrics, out_relu_y, big_scratch, stream);
    default: return hipErrorInvalidValue;
  }
}
