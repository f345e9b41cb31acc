// C ABI of libdaf: argument checks, plan construction, dispatch to the kernel launchers.
// Every check that does not need the GPU comes before the first HIP call.
#include <mutex>
#include <new>

#include "daf_internal.h"

namespace {

bool valid_width(int b) { return b == 1 || b == 2 || b == 4 || b == 8; }
bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct DeviceGuard {      // make the plan's device current for the duration of a call
  int prev = -1;
  bool switched = false;
  hipError_t enter(int dev) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != dev) {
      e = hipSetDevice(dev);
      switched = (e == hipSuccess);
    }
    return e;
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

}  // namespace

// Scratch memory of daf_quantize_pack_static: the per-tile and per-group (min, max) pairs of the
// two-pass route, for callers that cannot allocate.  One copy per GPU, held until the process
// ends.  In host code `scratch` is only a handle for hipGetSymbolAddress; the device address
// it yields (one per device) is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[DAF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, once looked up

// The address of `scratch` on the current device (looked up on the first call there).
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

bool daf_plan_needs_big_scratch(int64_t n, int32_t group_size, int64_t num_groups, int64_t* bytes) {
  constexpr int64_t kTile = 4096;
  if (group_size <= kTile) return false;
  if (group_size % kTile != 0 && num_groups != 1) return false;   // handled group by group instead
  const int64_t n_partials = (n + kTile - 1) / kTile;
  *bytes = (n_partials + num_groups) * 8;
  return true;
}

extern "C" {

int daf_rand_bits(void) { return 8; }

const char* daf_status_string(int status) {
  switch (status) {
    case DAF_OK: return "DAF_OK";
    case DAF_EINVAL: return "DAF_EINVAL: invalid argument";
    case DAF_EUNSUPPORTED: return "DAF_EUNSUPPORTED: unsupported group size, dtype or packed size";
    case DAF_ENOMEM: return "DAF_ENOMEM: allocation failed";
    case DAF_EDEVICE: return "DAF_EDEVICE: HIP call or kernel launch failed";
    case DAF_ETOOLARGE: return "DAF_ETOOLARGE: the tensor needs more scratch memory than the library's static buffer holds";
    default: return "unknown daf status";
  }
}

int daf_plan(const int64_t* shape, int ndim, int32_t group_size, const uint8_t* bits, int64_t n_bits,
             void* stream, daf_plan_t** out_plan) {
  if (out_plan == nullptr) return DAF_EINVAL;
  *out_plan = nullptr;
  if (shape == nullptr || bits == nullptr || ndim < 1) return DAF_EINVAL;
  int64_t n = 1;
  for (int d = 0; d < ndim; ++d) {
    if (shape[d] < 1) return DAF_EINVAL;
    if (n > INT64_MAX / shape[d]) return DAF_EUNSUPPORTED;
    n *= shape[d];
  }
  if (group_size < 32 || group_size % 32 != 0) return DAF_EUNSUPPORTED;
  const int64_t G = (n + group_size - 1) / group_size;
  if (n_bits != 1 && n_bits != G) return DAF_EINVAL;

  daf_plan_t* p = new (std::nothrow) daf_plan_t();
  if (p == nullptr) return DAF_ENOMEM;
  p->n = n;
  p->num_groups = G;
  p->group_size = group_size;
  p->d_bits = nullptr;
  p->d_off = nullptr;
  p->d_big_scratch = nullptr;
  p->d_scan = nullptr;
  p->scan_blocks = 0;
  p->pending = 0;
  {
    const int64_t full = n / group_size, tail = n - full * group_size;
    p->bound_words = full * ((int64_t)group_size * 8 / 32) + (tail * 8 + 31) / 32;
  }
  p->device = -1;
  p->output_cached = 0;
  int64_t big_bytes = 0;
  const bool big = daf_plan_needs_big_scratch(n, group_size, G, &big_bytes);

  if (n_bits == 1) {                     // uniform width: `bits` is a host pointer, no device work
    const int b = bits[0];
    if (!valid_width(b)) { delete p; return DAF_EINVAL; }
    const int64_t full = n / group_size, tail = n - full * group_size;
    const int64_t total = full * ((int64_t)group_size * b / 32) + (tail * b + 31) / 32;
    if (total >= (int64_t)1 << 32) { delete p; return DAF_EUNSUPPORTED; }
    p->uniform_bits = b;
    p->total_words = total;
    (void)hipGetDevice(&p->device);      // remembered when a device exists; harmless otherwise
    if (big && hipMalloc(&p->d_big_scratch, (size_t)big_bytes) != hipSuccess) {
      delete p;
      return DAF_ENOMEM;
    }
    *out_plan = p;
    return DAF_OK;
  }

  // per-group widths: device copy + device scan
  p->uniform_bits = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = DAF_OK;
  const int64_t n_blocks = daf_plan_scan_blocks(G);
  struct ScanResult { unsigned long long total; int bad; int pad; };   // (as in daf_plan_finish)
  // One device allocation holds the offsets, the scan's block sums (+ total and error flag) and
  // the plan's copy of the widths; the scan's result comes back through pinned host memory
  // (allocated once per thread): allocations, frees and a copy into pageable memory each cost
  // tens of microseconds, several times the three scan kernels together.
  static thread_local ScanResult* h_pinned = nullptr;
  ScanResult h = {0, 0, 0};
  do {
    if (hipGetDevice(&p->device) != hipSuccess) { rc = DAF_EDEVICE; break; }
    if (h_pinned == nullptr && hipHostMalloc(reinterpret_cast<void**>(&h_pinned), sizeof(ScanResult), hipHostMallocPortable) != hipSuccess) {
      h_pinned = nullptr;
      rc = DAF_ENOMEM;
      break;
    }
    const size_t off_bytes = (((size_t)G * sizeof(uint32_t)) + 15) & ~(size_t)15;
    const size_t sums_bytes = (((size_t)(n_blocks + 2) * sizeof(unsigned long long)) + 15) & ~(size_t)15;
    char* base = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&base), off_bytes + sums_bytes + (size_t)G) != hipSuccess) { rc = DAF_ENOMEM; break; }
    p->d_off = reinterpret_cast<uint32_t*>(base);          // the allocation's address: freed through d_off
    unsigned long long* d_sums = reinterpret_cast<unsigned long long*>(base + off_bytes);
    p->d_bits = reinterpret_cast<uint8_t*>(base + off_bytes + sums_bytes);
    if (big && hipMalloc(&p->d_big_scratch, (size_t)big_bytes) != hipSuccess) { rc = DAF_ENOMEM; break; }
    p->d_scan = d_sums;
    p->scan_blocks = n_blocks;
    unsigned long long* d_total = d_sums + n_blocks;
    int* d_bad = reinterpret_cast<int*>(d_sums + n_blocks + 1);
    if (daf_launch_plan_scan(bits, p->d_bits, G, n, group_size, p->d_off, d_sums, n_blocks, d_total, d_bad, st) != hipSuccess) { rc = DAF_EDEVICE; break; }
    if (hipMemcpyAsync(h_pinned, d_total, sizeof(ScanResult), hipMemcpyDeviceToHost, st) != hipSuccess) { rc = DAF_EDEVICE; break; }
    if (hipStreamSynchronize(st) != hipSuccess) { rc = DAF_EDEVICE; break; }
    h = *h_pinned;
    if (h.bad) { rc = DAF_EINVAL; break; }
    if (h.total >= 1ull << 32) { rc = DAF_EUNSUPPORTED; break; }
    p->total_words = (int64_t)h.total;
  } while (false);
  if (rc != DAF_OK) {
    daf_plan_destroy(p);
    return rc;
  }
  *out_plan = p;
  return DAF_OK;
}

namespace {
struct ScanResult { unsigned long long total; int bad; int pad; };
}

int daf_plan_update(daf_plan_t* plan, const uint8_t* bits, void* stream) {
  if (plan == nullptr || bits == nullptr) return DAF_EINVAL;
  if (plan->uniform_bits != 0 || plan->d_scan == nullptr) return DAF_EINVAL;   // per-group-width plans only
  if (plan->bound_words >= (int64_t)1 << 32) return DAF_EUNSUPPORTED;          // offsets are 32-bit words
  unsigned long long* d_total = plan->d_scan + plan->scan_blocks;
  int* d_bad = reinterpret_cast<int*>(plan->d_scan + plan->scan_blocks + 1);
  if (daf_launch_plan_scan(bits, plan->d_bits, plan->num_groups, plan->n, plan->group_size, plan->d_off, plan->d_scan,
                           plan->scan_blocks, d_total, d_bad, static_cast<hipStream_t>(stream)) != hipSuccess)
    return DAF_EDEVICE;
  plan->pending = 1;
  plan->total_words = plan->bound_words;
  return DAF_OK;
}

int daf_plan_finish(daf_plan_t* plan, void* stream) {
  if (plan == nullptr) return DAF_EINVAL;
  if (!plan->pending) return DAF_OK;
  ScanResult h = {0, 0, 0};
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&h, plan->d_scan + plan->scan_blocks, sizeof(ScanResult), hipMemcpyDeviceToHost, st) != hipSuccess)
    return DAF_EDEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return DAF_EDEVICE;
  plan->pending = 0;
  plan->total_words = (int64_t)h.total;      // with invalid widths counted as 8 bits: the layout the kernels used
  return h.bad ? DAF_EINVAL : DAF_OK;
}

int64_t daf_plan_packed_words_bound(const daf_plan_t* plan) { return plan ? plan->bound_words : -1; }

int64_t daf_plan_num_elements(const daf_plan_t* plan) { return plan ? plan->n : -1; }
int64_t daf_plan_num_groups(const daf_plan_t* plan) { return plan ? plan->num_groups : -1; }
int64_t daf_plan_packed_words(const daf_plan_t* plan) { return plan ? plan->total_words : -1; }
int32_t daf_plan_group_size(const daf_plan_t* plan) { return plan ? plan->group_size : -1; }
int32_t daf_plan_uniform_bits(const daf_plan_t* plan) { return plan ? plan->uniform_bits : -1; }

int daf_plan_set_output_cached(daf_plan_t* plan, int cached) {
  if (plan == nullptr || (cached != 0 && cached != 1)) return DAF_EINVAL;
  plan->output_cached = cached;
  return DAF_OK;
}

int daf_plan_quantize_route(const daf_plan_t* plan, daf_dtype_t dtype) {
  if (plan == nullptr) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  return daf_quantize_route(plan, (int)dtype);
}

int daf_plan_copy_offsets(const daf_plan_t* plan, uint32_t* out_off) {
  if (plan == nullptr || out_off == nullptr) return DAF_EINVAL;
  if (plan->uniform_bits) {
    const uint32_t wpg = (uint32_t)((int64_t)plan->group_size * plan->uniform_bits / 32);
    for (int64_t g = 0; g < plan->num_groups; ++g) out_off[g] = (uint32_t)g * wpg;
    return DAF_OK;
  }
  DeviceGuard guard;
  if (guard.enter(plan->device) != hipSuccess) return DAF_EDEVICE;
  if (hipMemcpy(out_off, plan->d_off, (size_t)plan->num_groups * sizeof(uint32_t), hipMemcpyDeviceToHost) != hipSuccess)
    return DAF_EDEVICE;
  return DAF_OK;
}

void daf_plan_destroy(daf_plan_t* plan) {
  if (plan == nullptr) return;
  if (plan->d_off) (void)hipFree(plan->d_off);            // one allocation: offsets, scan scratch, widths
  if (plan->d_big_scratch) (void)hipFree(plan->d_big_scratch);
  delete plan;
}

int daf_quantize_pack(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, uint64_t seed,
                      uint32_t* out_words, float* out_min, float* out_scale, void* stream) {
  if (plan == nullptr || x == nullptr || out_words == nullptr || out_min == nullptr || out_scale == nullptr)
    return DAF_EINVAL;
  if (!aligned(x, 16) || !aligned(out_words, 4) || !aligned(out_min, 4) || !aligned(out_scale, 4)) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  const hipError_t e = daf_launch_quantize_pack(plan, x, (int)dtype, seed, out_words, out_min, out_scale, nullptr,
                                                nullptr, nullptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_quantize_pack_static(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, uint64_t seed,
                             uint32_t* out_words, float* out_min, float* out_scale, void* stream) {
  if (plan == nullptr || x == nullptr || out_words == nullptr || out_min == nullptr || out_scale == nullptr)
    return DAF_EINVAL;
  if (!aligned(x, 16) || !aligned(out_words, 4) || !aligned(out_min, 4) || !aligned(out_scale, 4)) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  void* ptr = nullptr;
  if (daf_quantize_route(plan, (int)dtype) == DAF_ROUTE_TWO_PASS) {     // the only route with scratch memory
    int64_t bytes = 0;
    (void)daf_plan_needs_big_scratch(plan->n, plan->group_size, plan->num_groups, &bytes);
    if (bytes > (int64_t)DAF_STATIC_SCRATCH_BYTES) return DAF_ETOOLARGE;
    if (static_scratch(&ptr) != hipSuccess) return DAF_EDEVICE;
  }
  const hipError_t e = daf_launch_quantize_pack(plan, x, (int)dtype, seed, out_words, out_min, out_scale, nullptr,
                                                nullptr, ptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_quantize_pack_batch(const daf_quantize_item_t* items, int32_t n_items, daf_dtype_t dtype, void* stream) {
  if (items == nullptr || n_items < 1) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  for (int32_t i = 0; i < n_items; ++i) {
    const daf_quantize_item_t& it = items[i];
    if (it.plan == nullptr || it.x == nullptr || it.out_words == nullptr || it.out_min == nullptr ||
        it.out_scale == nullptr)
      return DAF_EINVAL;
    if (!aligned(it.x, 16) || !aligned(it.out_words, 4) || !aligned(it.out_min, 4) || !aligned(it.out_scale, 4))
      return DAF_EINVAL;
  }
  const hipError_t e = daf_launch_quantize_pack_batch(items, n_items, (int)dtype, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_unpack_dequantize_batch(const daf_dequantize_item_t* items, int32_t n_items, daf_dtype_t dtype, void* stream) {
  if (items == nullptr || n_items < 1) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  for (int32_t i = 0; i < n_items; ++i) {
    const daf_dequantize_item_t& it = items[i];
    if (it.plan == nullptr || it.words == nullptr || it.min == nullptr || it.scale == nullptr || it.out_x == nullptr)
      return DAF_EINVAL;
    if (!aligned(it.out_x, 16) || !aligned(it.words, 4) || !aligned(it.min, 4) || !aligned(it.scale, 4))
      return DAF_EINVAL;
    if (it.plan->uniform_bits && it.bits != nullptr) return DAF_EINVAL;
  }
  const hipError_t e = daf_launch_unpack_dequantize_batch(items, n_items, (int)dtype, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_relu_quantize_pack(const daf_plan_t* plan, const void* z, daf_dtype_t dtype, uint64_t seed, void* out_y,
                           uint32_t* out_words, float* out_min, float* out_scale, void* stream) {
  if (plan == nullptr || z == nullptr || out_y == nullptr || out_words == nullptr || out_min == nullptr ||
      out_scale == nullptr)
    return DAF_EINVAL;
  if (!aligned(z, 16) || !aligned(out_y, 16) || !aligned(out_words, 4) || !aligned(out_min, 4) ||
      !aligned(out_scale, 4))
    return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  if (!daf_quantize_reads_once(plan)) return DAF_EUNSUPPORTED;     // the group's statistics need a pass of their own
  if (out_y != z) {                                                // in place, or not overlapping at all
    const int64_t bytes = plan->n * (dtype == DAF_F32 ? 4 : 2);
    const char* a = static_cast<const char*>(z);
    const char* b = static_cast<const char*>(out_y);
    if (a < b + bytes && b < a + bytes) return DAF_EINVAL;
  }
  const hipError_t e = daf_launch_quantize_pack(plan, z, (int)dtype, seed, out_words, out_min, out_scale, nullptr,
                                                out_y, nullptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_linear_quantize_pack(const daf_plan_t* plan, const void* x, const void* weight, int64_t N, int64_t K,
                             daf_dtype_t dtype, uint64_t seed, void* out_y, uint32_t* out_words, float* out_min,
                             float* out_scale, void* stream) {
  if (plan == nullptr || x == nullptr || weight == nullptr || out_y == nullptr || N < 1 || K < 1) return DAF_EINVAL;
  // all three packed outputs, or none of them (the product alone)
  const bool product_only = out_words == nullptr && out_min == nullptr && out_scale == nullptr;
  if (!product_only && (out_words == nullptr || out_min == nullptr || out_scale == nullptr)) return DAF_EINVAL;
  if (!aligned(x, 16) || !aligned(weight, 16) || !aligned(out_y, 16) || !aligned(out_words, 4) ||
      !aligned(out_min, 4) || !aligned(out_scale, 4))
    return DAF_EINVAL;
  if (plan->n % N != 0) return DAF_EINVAL;
  if (!daf_linear_quantize_supported(plan, N, K, (int)dtype)) return DAF_EUNSUPPORTED;
  const hipError_t e = daf_launch_linear_quantize_pack(plan, x, weight, N, K, (int)dtype, seed, out_y, out_words,
                                                       out_min, out_scale, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_linear_tile_of_workgroup(int32_t id, int32_t tiles_m, int32_t tiles_n, int32_t* tile_m, int32_t* tile_n) {
  if (tile_m == nullptr || tile_n == nullptr || tiles_m < 1 || tiles_n < 1 || id < 0 ||
      (int64_t)id >= (int64_t)tiles_m * tiles_n)
    return DAF_EINVAL;
  int m, n;
  daf_linear_tile_map(id, tiles_m, tiles_n, &m, &n);
  *tile_m = m;
  *tile_n = n;
  return DAF_OK;
}

int daf_quantize_pack_metrics(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, uint64_t seed,
                              uint32_t* out_words, float* out_min, float* out_scale, float* out_metrics,
                              void* stream) {
  if (plan == nullptr || x == nullptr || out_words == nullptr || out_min == nullptr || out_scale == nullptr ||
      out_metrics == nullptr)
    return DAF_EINVAL;
  if (!aligned(x, 16) || !aligned(out_words, 4) || !aligned(out_min, 4) || !aligned(out_scale, 4) ||
      !aligned(out_metrics, 4))
    return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  if (!daf_quantize_reads_once(plan)) return DAF_EUNSUPPORTED;     // the group's statistics need a pass of their own
  const hipError_t e = daf_launch_quantize_pack(plan, x, (int)dtype, seed, out_words, out_min, out_scale,
                                                out_metrics, nullptr, nullptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_unpack_dequantize(const daf_plan_t* plan, const uint32_t* words, const float* min, const float* scale,
                          const uint8_t* bits, void* out_x, daf_dtype_t dtype, void* stream) {
  if (plan == nullptr || words == nullptr || min == nullptr || scale == nullptr || out_x == nullptr) return DAF_EINVAL;
  if (!aligned(out_x, 16) || !aligned(words, 4) || !aligned(min, 4) || !aligned(scale, 4)) return DAF_EINVAL;
  if (plan->uniform_bits && bits != nullptr) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  const uint8_t* d_bits = bits ? bits : plan->d_bits;
  const hipError_t e = daf_launch_unpack_dequantize(plan, words, min, scale, d_bits, out_x, (int)dtype, nullptr,
                                                    static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_unpack_relu_backward(const daf_plan_t* plan, const uint32_t* words, const float* min, const float* scale,
                             const uint8_t* bits, const void* grad_y, void* out_grad_z, daf_dtype_t dtype,
                             void* stream) {
  if (plan == nullptr || words == nullptr || min == nullptr || scale == nullptr || grad_y == nullptr ||
      out_grad_z == nullptr)
    return DAF_EINVAL;
  if (!aligned(out_grad_z, 16) || !aligned(grad_y, 16) || !aligned(words, 4) || !aligned(min, 4) ||
      !aligned(scale, 4))
    return DAF_EINVAL;
  if (plan->uniform_bits && bits != nullptr) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  if (out_grad_z != grad_y) {                                      // in place, or not overlapping at all
    const int64_t bytes = plan->n * (dtype == DAF_F32 ? 4 : 2);
    const char* a = static_cast<const char*>(grad_y);
    const char* b = static_cast<const char*>(out_grad_z);
    if (a < b + bytes && b < a + bytes) return DAF_EINVAL;
  }
  const uint8_t* d_bits = bits ? bits : plan->d_bits;
  const hipError_t e = daf_launch_unpack_dequantize(plan, words, min, scale, d_bits, out_grad_z, (int)dtype, grad_y,
                                                    static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int64_t daf_unpack_matmul_workspace_bytes(const daf_plan_t* plan, int64_t N, int64_t K) {
  if (plan == nullptr || N <= 0 || K <= 0 || plan->n % K != 0) return -1;
  const int64_t M = plan->n / K;
  if (!daf_unpack_matmul_shape_ok(M, N, K, plan->group_size)) return -1;
  return daf_unpack_matmul_workspace_size(M, N, K);
}

int daf_unpack_matmul_grad_weight(const daf_plan_t* plan, const uint32_t* words, const float* min, const float* scale,
                                  const uint8_t* bits, const void* grad_y, int64_t N, int64_t K, daf_dtype_t dtype,
                                  float* out_grad_w, void* workspace, void* stream) {
  if (plan == nullptr || words == nullptr || min == nullptr || scale == nullptr || grad_y == nullptr ||
      out_grad_w == nullptr)
    return DAF_EINVAL;
  if (N <= 0 || K <= 0 || plan->n % K != 0) return DAF_EINVAL;
  if (!aligned(grad_y, 16) || !aligned(out_grad_w, 16) || !aligned(words, 4) || !aligned(min, 4) ||
      !aligned(scale, 4) || !aligned(workspace, 16))
    return DAF_EINVAL;
  if (plan->uniform_bits && bits != nullptr) return DAF_EINVAL;
  if (dtype != DAF_F16 && dtype != DAF_BF16 && dtype != DAF_F32) return DAF_EUNSUPPORTED;
  const int64_t M = plan->n / K;
  if (!daf_unpack_matmul_shape_ok(M, N, K, plan->group_size)) return DAF_EUNSUPPORTED;
  if (plan->total_words >= (int64_t)1 << 30) return DAF_EUNSUPPORTED;   // 32-bit byte offsets into the words
  if (daf_unpack_matmul_workspace_size(M, N, K) > 0 && workspace == nullptr) return DAF_EINVAL;
  const uint8_t* d_bits = bits ? bits : plan->d_bits;
  const hipError_t e = daf_launch_unpack_matmul(plan, words, min, scale, d_bits, grad_y, N, K, (int)dtype, out_grad_w,
                                                static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int64_t daf_minmax_workspace_bytes(void) { return daf_minmax_workspace_size(); }

int daf_minmax_workspace_init(void* workspace, void* stream) {
  if (workspace == nullptr || !aligned(workspace, 16)) return DAF_EINVAL;
  return daf_launch_minmax_workspace_init(workspace, static_cast<hipStream_t>(stream)) == hipSuccess ? DAF_OK
                                                                                                    : DAF_EDEVICE;
}

int daf_minmax(const void* x, daf_dtype_t dtype, int64_t n, int method, void* workspace, float* out_minmax,
               void* stream) {
  if (x == nullptr || workspace == nullptr || out_minmax == nullptr || n < 1) return DAF_EINVAL;
  if (!aligned(x, 16) || !aligned(workspace, 16) || !aligned(out_minmax, 4)) return DAF_EINVAL;
  if (method != DAF_REDUCE_TWO_PASS && method != DAF_REDUCE_ATOMIC) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  const hipError_t e = daf_launch_minmax(x, (int)dtype, n, method, workspace, out_minmax,
                                         static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_group_minmax(const daf_plan_t* plan, const void* x, daf_dtype_t dtype, float* out_min, float* out_max,
                     void* stream) {
  if (plan == nullptr || x == nullptr || out_min == nullptr || out_max == nullptr) return DAF_EINVAL;
  if (!aligned(x, 16) || !aligned(out_min, 4) || !aligned(out_max, 4)) return DAF_EINVAL;
  if (dtype != DAF_F32 && dtype != DAF_F16 && dtype != DAF_BF16) return DAF_EUNSUPPORTED;
  const hipError_t e = daf_launch_group_minmax(plan, x, (int)dtype, out_min, out_max, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int64_t daf_select_bits_workspace_bytes(int64_t num_groups) {
  return num_groups < 1 ? -1 : daf_select_bits_workspace_size(num_groups);
}

int daf_select_bits(const float* group_min, const float* group_max, int64_t num_groups, const uint8_t* classes,
                    int32_t n_classes, uint8_t* out_bits, void* workspace, void* stream) {
  if (group_min == nullptr || group_max == nullptr || classes == nullptr || out_bits == nullptr ||
      workspace == nullptr || num_groups < 1 || n_classes < 1 || n_classes > 4)
    return DAF_EINVAL;
  if (!aligned(group_min, 4) || !aligned(group_max, 4) || !aligned(workspace, 16)) return DAF_EINVAL;
  for (int c = 0; c < n_classes; ++c)
    if (!valid_width(classes[c])) return DAF_EINVAL;
  if (num_groups >= (int64_t)1 << 32) return DAF_EUNSUPPORTED;
  const hipError_t e = daf_launch_select_bits(group_min, group_max, nullptr, 0, num_groups, classes, n_classes, out_bits,
                                              workspace, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

int daf_select_bits_from_scale(const float* group_scale, const uint8_t* group_bits, int32_t uniform_bits,
                               int64_t num_groups, const uint8_t* classes, int32_t n_classes, uint8_t* out_bits,
                               void* workspace, void* stream) {
  if (group_scale == nullptr || classes == nullptr || out_bits == nullptr || workspace == nullptr || num_groups < 1 ||
      n_classes < 1 || n_classes > 4)
    return DAF_EINVAL;
  if (group_bits == nullptr && !valid_width((uint8_t)uniform_bits)) return DAF_EINVAL;
  if (!aligned(group_scale, 4) || !aligned(workspace, 16)) return DAF_EINVAL;
  for (int c = 0; c < n_classes; ++c)
    if (!valid_width(classes[c])) return DAF_EINVAL;
  if (num_groups >= (int64_t)1 << 32) return DAF_EUNSUPPORTED;
  const hipError_t e = daf_launch_select_bits(group_scale, nullptr, group_bits, uniform_bits, num_groups, classes,
                                              n_classes, out_bits, workspace, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DAF_OK : DAF_EDEVICE;
}

}  // extern "C"
