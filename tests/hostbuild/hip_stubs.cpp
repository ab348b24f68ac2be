// CPU stand-ins for the HIP runtime calls and kernel launchers the host library uses, so that
// oxy_pool.cpp and oxy_sched.cpp can be compiled with gcc under AddressSanitizer /
// UndefinedBehaviorSanitizer and run on a machine without a GPU.  "Device" memory is host
// memory here; launches do nothing.  oxy_stub_fail_next(skip, k) makes k device-facing calls fail
// after `skip` more successful ones, which is how the tests force the error paths from the host.
#include "../../paper_2603_14371_amd/csrc/oxy_internal.h"

#include <cstdlib>
#include <cstring>

static int g_fail_next = 0, g_fail_skip = 0;
static long g_calls = 0;
// after `skip` further successful calls, the next k device-facing calls fail
extern "C" void oxy_stub_fail_next(int skip, int k) { g_fail_skip = skip, g_fail_next = k; }
extern "C" long oxy_stub_calls() { return g_calls; }

static hipError_t outcome() {
  ++g_calls;
  if (g_fail_skip > 0) {
    --g_fail_skip;
    return hipSuccess;
  }
  if (g_fail_next > 0) {
    --g_fail_next;
    return hipErrorUnknown;
  }
  return hipSuccess;
}

extern "C" {
const char* hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "stubbed failure"; }
hipError_t hipHostMalloc(void** p, size_t n, unsigned int) {
  *p = malloc(n ? n : 1);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostFree(void* p) {
  free(p);
  return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) {
  *e = (hipEvent_t)malloc(8);
  return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t e) {
  free((void*)e);
  return hipSuccess;
}
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return outcome(); }
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) {
  hipError_t e = outcome();
  if (e == hipSuccess) memcpy(dst, src, n);   // the sanitizer checks both ranges
  return e;
}
// recorded launch sequences: a stream, a graph and an instantiated graph are small heap objects,
// so that the sanitizer sees every leak, double free and use after free of the host logic
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
  *s = (hipStream_t)malloc(8);
  return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t s) {
  free((void*)s);
  return hipSuccess;
}
hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { return outcome(); }
hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t* g) {
  *g = (hipGraph_t)malloc(8);
  return hipSuccess;
}
hipError_t hipGraphDestroy(hipGraph_t g) {
  free((void*)g);
  return hipSuccess;
}
hipError_t hipGraphInstantiate(hipGraphExec_t* x, hipGraph_t, hipGraphNode_t*, char*, size_t) {
  hipError_t e = outcome();
  if (e == hipSuccess) *x = (hipGraphExec_t)malloc(8);
  return e;
}
hipError_t hipGraphExecDestroy(hipGraphExec_t x) {
  free((void*)x);
  return hipSuccess;
}
hipError_t hipGraphExecUpdate(hipGraphExec_t x, hipGraph_t, hipGraphNode_t*,
                              hipGraphExecUpdateResult* res) {
  *(volatile char*)x;   // must still be alive
  hipError_t e = outcome();
  *res = e == hipSuccess ? hipGraphExecUpdateSuccess : hipGraphExecUpdateError;
  return e;
}
hipError_t hipGraphLaunch(hipGraphExec_t x, hipStream_t) {
  *(volatile char*)x;
  return outcome();
}
hipError_t hipMemsetAsync(void* dst, int v, size_t n, hipStream_t) {
  hipError_t e = outcome();
  if (e == hipSuccess) memset(dst, v, n);
  return e;
}
}

namespace oxy {
hipError_t launch_append(const void*, const void*, const int32_t*, int32_t, void*, hipStream_t) {
  return outcome();
}
hipError_t launch_append_inline(const void*, const void*, const InlineIds&, int32_t, int32_t, void*,
                                int32_t, size_t, size_t, hipStream_t) {
  return outcome();
}
hipError_t launch_gather_inline(const void*, const InlineIds&, int32_t, void*, void*, hipStream_t) {
  return outcome();
}
hipError_t launch_attention(const AttnArgs&, hipStream_t) { return outcome(); }
hipError_t static_scratch(uint16_t** part_acc, float** part_ml) {
  static char buf[64];
  *part_acc = (uint16_t*)buf;
  *part_ml = (float*)buf;
  return hipSuccess;
}
hipError_t launch_attention_work(const AttnArgs&, hipStream_t, hipEvent_t, hipEvent_t) {
  return outcome();
}
hipError_t launch_merge_append(const AttnArgs&, const AppendArgs*, hipStream_t, hipEvent_t,
                               hipEvent_t) {
  return outcome();
}
}  // namespace oxy
