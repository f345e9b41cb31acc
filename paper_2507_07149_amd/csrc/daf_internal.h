// Internal declarations shared by the translation units of libdaf (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "daf.h"

struct daf_plan_s {
  int64_t n;             // elements
  int64_t num_groups;    // G = ceil(n / group_size)
  int64_t total_words;   // packed size
  int32_t group_size;
  int32_t uniform_bits;  // shared width, or 0 when widths are per group
  int device;            // HIP device the plan's memory lives on
  int32_t output_cached; // unpack+dequantize output: 0 streaming stores (default), 1 cached stores
  uint8_t* d_bits;       // G widths (device), mixed plans only; lives inside d_off's allocation
  uint32_t* d_off;       // G word offsets (device), mixed plans only; the address that is freed
  void* d_big_scratch;   // groups longer than a 4096-element tile: one (min, max) pair per tile and
                         // per group, written by the quantize call's first pass (else null)
  unsigned long long* d_scan;  // mixed plans: the scan's block sums, then the total and the invalid-width flag
  int64_t scan_blocks;
  int64_t bound_words;   // packed size if every group had 8 bits: what total_words reads while an
                         // update's exact size has not been fetched (pending != 0)
  int32_t pending;
};

// True when the plan's groups are longer than a tile and tile-aligned (or there is one group),
// i.e. when daf_quantize_pack takes the two-pass route; bytes of scratch it then needs.
bool daf_plan_needs_big_scratch(int64_t n, int32_t group_size, int64_t num_groups, int64_t* bytes);

// True when daf_quantize_pack reads the activation once for this plan (no statistics pass first):
// the fused variants that write a second output in the same pass exist for such plans only.
bool daf_quantize_reads_once(const daf_plan_t* plan);

// The kernels daf_quantize_pack uses for the plan's whole groups: a value of daf_route_t, -1 for an
// unknown dtype.  A host computation.
int daf_quantize_route(const daf_plan_t* plan, int dtype);

// Launchers.  Each returns hipSuccess or the first HIP error.
// src_bits: the caller's widths; plan_bits: the plan's copy, written by the scan with every width
// outside {1,2,4,8} replaced by 8 (and *d_bad set).  No value needs clearing beforehand.
hipError_t daf_launch_plan_scan(const uint8_t* src_bits, uint8_t* plan_bits, int64_t num_groups, int64_t n,
                                int32_t group_size, uint32_t* d_off, unsigned long long* d_block_sums, int64_t n_blocks,
                                unsigned long long* d_total, int* d_bad, hipStream_t stream);
int64_t daf_plan_scan_blocks(int64_t num_groups);

// out_metrics: null, or 3 floats per group (sum (x-xhat)^2, sum x^2, rounding variance); not with groups longer than a tile.
// out_relu_y: null, or the buffer that receives max(x, +0), which is then what gets quantized (may be x
// itself); not together with out_metrics, not with groups longer than a tile.
// big_scratch: null = the plan's own scratch; else device memory of at least the size
// daf_plan_needs_big_scratch reports, used by the two-pass route in its place.
hipError_t daf_launch_quantize_pack(const daf_plan_t* plan, const void* x, int dtype, uint64_t seed,
                                    uint32_t* out_words, float* out_min, float* out_scale, float* out_metrics,
                                    void* out_relu_y, void* big_scratch, hipStream_t stream);

// Weight gradient straight from the packed activation (unpack_matmul.hip).  The plan's tensor is
// read as [n / K, K]; out is [N, K] binary32; workspace holds daf_unpack_matmul_workspace_size bytes.
int64_t daf_unpack_matmul_workspace_size(int64_t M, int64_t N, int64_t K);   // bytes (0: none needed)
bool daf_unpack_matmul_shape_ok(int64_t M, int64_t N, int64_t K, int32_t gs);
hipError_t daf_launch_unpack_matmul(const daf_plan_t* p, const uint32_t* words, const float* mn, const float* scale,
                                    const uint8_t* d_bits, const void* grad_y, int64_t N, int64_t K, int dtype,
                                    float* out, float* workspace, hipStream_t stream);

// One call for several tensors of one dtype (daf_quantize_item_t / daf_dequantize_item_t: daf.h).
hipError_t daf_launch_quantize_pack_batch(const daf_quantize_item_t* items, int32_t n_items, int dtype,
                                          hipStream_t stream);
hipError_t daf_launch_unpack_dequantize_batch(const daf_dequantize_item_t* items, int32_t n_items, int dtype,
                                              hipStream_t stream);

// relu_grad_y: null, or the gradient of y = max(z, 0): out_x then receives (xhat > 0) ? grad_y : +0
hipError_t daf_launch_unpack_dequantize(const daf_plan_t* plan, const uint32_t* words, const float* mn,
                                        const float* scale, const uint8_t* d_bits, void* out_x, int dtype,
                                        const void* relu_grad_y, hipStream_t stream);

int64_t daf_minmax_workspace_size(void);
hipError_t daf_launch_minmax_workspace_init(void* workspace, hipStream_t stream);
hipError_t daf_launch_minmax(const void* x, int dtype, int64_t n, int method, void* workspace, float* out_minmax,
                             hipStream_t stream);

hipError_t daf_launch_group_minmax(const daf_plan_t* plan, const void* x, int dtype, float* out_min, float* out_max,
                                   hipStream_t stream);
int64_t daf_select_bits_workspace_size(int64_t num_groups);
// y = x W^T with quantize+pack of y in the tile epilogue (linear_quantize.hip).  `supported` is a host
// check of shapes, group size and dtype; the launcher assumes it holds.
bool daf_linear_quantize_supported(const daf_plan_t* plan, int64_t N, int64_t K, int dtype);
// The output tile (256 x 256) that workgroup `id` of the launch computes; a host copy of the kernel's own map.
void daf_linear_tile_map(int id, int tiles_m, int tiles_n, int* tm, int* tn);
hipError_t daf_launch_linear_quantize_pack(const daf_plan_t* plan, const void* x, const void* w, int64_t N, int64_t K,
                                           int dtype, uint64_t seed, void* y, uint32_t* words, float* mn, float* sc,
                                           hipStream_t stream);

// gmax != null: ranges are gmax - gmin.  gmax == null: gmin holds scales, ranges are scale * (2^b - 1)
// with b = prev_bits[g] (device) or prev_uniform when prev_bits is null.
hipError_t daf_launch_select_bits(const float* gmin, const float* gmax, const uint8_t* prev_bits, int32_t prev_uniform,
                                  int64_t num_groups, const uint8_t* classes, int n_classes, uint8_t* out_bits,
                                  void* workspace, hipStream_t stream);
