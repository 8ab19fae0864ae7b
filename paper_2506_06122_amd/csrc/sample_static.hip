// rollout_sample_static: the stand-alone sampler for callers that cannot allocate device memory
// (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  Same kernels
// as rollout_sample; what that entry point allocates per call - the per-row parameter arrays and
// the sweeps' partial results (kernels.h, SampleRows) - lives here in one file-scope device
// array of fixed size, so the call allocates nothing, copies nothing between host and device
// and does not synchronise: it only enqueues kernels on the caller's stream.
#include <mutex>
#include <string>

#include "../../include/rollout.h"
#include "kernels.h"

namespace {

constexpr int kMaxRows = ROLLOUT_SAMPLE_STATIC_MAX_ROWS;
constexpr int kMaxDevices = 64;

// layout of the scratch array (byte offsets, each a multiple of 256)
constexpr size_t kOffInvTemp = 0;                                                  // float [kMaxRows]
constexpr size_t kOffTopP = kOffInvTemp + sizeof(float) * kMaxRows;                // float [kMaxRows]
constexpr size_t kOffPartMax = kOffTopP + sizeof(float) * kMaxRows;                // float [kMaxRows][kSampleParts]
constexpr size_t kOffSegSums = kOffPartMax + sizeof(float) * kMaxRows * kSampleParts;  // u64 [kMaxRows][kSampleSegments]
constexpr size_t kScratchBytes = kOffSegSums + sizeof(unsigned long long) * kMaxRows * kSampleSegments;
static_assert(kOffTopP % 256 == 0 && kOffPartMax % 256 == 0 && kOffSegSums % 256 == 0, "256-byte aligned parts");

// One copy per GPU the library runs on, held until the process ends (about 2.2 MB).  In host
// code this name is only a handle for hipGetSymbolAddress: the address a kernel can use is
// looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};

__global__ void fill_params_kernel(float* inv_temp, float* top_p, float inv_t, float p, int rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) {
    inv_temp[i] = inv_t;
    top_p[i] = p;
  }
}

thread_local std::string g_error;

int set_error(int code, const std::string& msg) {
  g_error = msg;
  return code;
}

// device address of this device's copy of `scratch`; looked up on the first call per device
int scratch_for_current_device(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return set_error(ROLLOUT_E_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return set_error(ROLLOUT_E_HIP, "device index out of range");
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return set_error(ROLLOUT_E_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = (unsigned char*)g_scratch_ptr[dev];
  return ROLLOUT_OK;
}

}  // namespace

extern "C" {

const char* rollout_sample_static_error(void) { return g_error.c_str(); }

int rollout_sample_static_prepare(void) {
  unsigned char* p = nullptr;
  return scratch_for_current_device(&p);
}

int rollout_sample_static(const float* logits, int32_t rows, int32_t vocab, float temperature, float top_p,
                          const uint32_t* uniforms, const int32_t* forced, void* hip_stream, int32_t* tokens,
                          float* logprobs, uint64_t* weight_sums) {
  if (!logits || rows < 0 || vocab < 1 || vocab > 262144 || !uniforms || !tokens || !logprobs)
    return set_error(ROLLOUT_E_INVAL, "bad argument");
  if (rows > kMaxRows)
    return set_error(ROLLOUT_E_INVAL, "rows exceeds ROLLOUT_SAMPLE_STATIC_MAX_ROWS (" + std::to_string(kMaxRows) + ")");
  if (!(temperature > 0.f) || !(temperature <= 3.0e38f) || !(top_p >= 0.f))
    return set_error(ROLLOUT_E_INVAL, "bad sampling parameters");
  if (rows == 0) return ROLLOUT_OK;
  unsigned char* base = nullptr;
  const int rc = scratch_for_current_device(&base);
  if (rc != ROLLOUT_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  float* inv_temp = (float*)(base + kOffInvTemp);
  float* tp = (float*)(base + kOffTopP);
  // nothing in the array has to start at zero: every element a kernel reads was written earlier in
  // the same call (the parameters here, the partial results by the sweeps before the selection)
  fill_params_kernel<<<(rows + 255) / 256, 256, 0, s>>>(inv_temp, tp, 1.0f / temperature, top_p, rows);
  SampleRows sr{};
  sr.logits = logits;
  sr.inv_temp = inv_temp;
  sr.top_p = tp;
  sr.uniforms = uniforms;
  sr.forced = forced;
  sr.tokens = tokens;
  sr.logprobs = logprobs;
  sr.weight_sums = (unsigned long long*)weight_sums;
  sr.part_max = (float*)(base + kOffPartMax);
  sr.seg_sums = (unsigned long long*)(base + kOffSegSums);
  launch_sample(sr, rows, vocab, s);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(ROLLOUT_E_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
  return ROLLOUT_OK;
}

}  // extern "C"
