// Process-wide state behind the launchers: the tuning / testing switches and the cached device facts.
// Nothing of the method lives here.
#include <cstdlib>
#include <cstring>

#include <mutex>

#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include "st_internal.h"
#include "st_testing.h"

namespace st {
namespace {

int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  return e ? atoi(e) : dflt;
}

Knobs knobs_from_env() {
  Knobs k;
  k.fwd_fast = env_int("ST_FWD_FAST", k.fwd_fast);
  k.dq_fast = env_int("ST_DQ_FAST", k.dq_fast);
  k.dkv_fast = env_int("ST_DKV_FAST", k.dkv_fast);
  k.dkv_queue = env_int("ST_DKV_QUEUE", k.dkv_queue);
  k.fwd_wq = env_int("ST_FWD_WQ", k.fwd_wq);
  k.fwd_pipe = env_int("ST_FWD_PIPE", k.fwd_pipe);
  if (const char* e = getenv("ST_FWD_GAP")) {
    const float g = (float)atof(e);
    if (g >= 0.f && g <= 64.f) k.fwd_gap = g;
  }
  return k;
}

// ---- number of XCDs of a HIP device: the HSA agent with the same PCI address tells ----
struct XccQuery {
  uint32_t domain, bdf;   // PCI address looked for
  int xcds;               // result, 0 = not found
};

hsa_status_t visit_agent(hsa_agent_t agent, void* data) {
  XccQuery* q = (XccQuery*)data;
  hsa_device_type_t type;
  if (hsa_agent_get_info(agent, HSA_AGENT_INFO_DEVICE, &type) != HSA_STATUS_SUCCESS || type != HSA_DEVICE_TYPE_GPU)
    return HSA_STATUS_SUCCESS;
  uint32_t bdf = 0, domain = 0, xcc = 0;
  if (hsa_agent_get_info(agent, (hsa_agent_info_t)HSA_AMD_AGENT_INFO_BDFID, &bdf) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
  if (hsa_agent_get_info(agent, (hsa_agent_info_t)HSA_AMD_AGENT_INFO_DOMAIN, &domain) != HSA_STATUS_SUCCESS) domain = q->domain;
  if (bdf != q->bdf || domain != q->domain) return HSA_STATUS_SUCCESS;
  if (hsa_agent_get_info(agent, (hsa_agent_info_t)HSA_AMD_AGENT_INFO_NUM_XCC, &xcc) == HSA_STATUS_SUCCESS && xcc >= 1)
    q->xcds = (int)xcc;
  return HSA_STATUS_INFO_BREAK;
}

int query_xcds(int dev) {
  int domain = 0, bus = 0, device = 0;
  if (hipDeviceGetAttribute(&domain, hipDeviceAttributePciDomainID, dev) != hipSuccess ||
      hipDeviceGetAttribute(&bus, hipDeviceAttributePciBusId, dev) != hipSuccess ||
      hipDeviceGetAttribute(&device, hipDeviceAttributePciDeviceId, dev) != hipSuccess)
    return 0;
  if (hsa_init() != HSA_STATUS_SUCCESS) return 0;        // reference counted; the HIP runtime holds it open already
  XccQuery q{(uint32_t)domain, (uint32_t)((bus << 8) | (device << 3)), 0};   // BDF with function 0
  (void)hsa_iterate_agents(visit_agent, &q);
  (void)hsa_shut_down();
  return q.xcds;
}

constexpr int kMaxDevices = 64;
std::mutex g_dev_mu;
DeviceInfo g_dev[kMaxDevices];
bool g_dev_known[kMaxDevices];

}  // namespace

Knobs& knobs() {
  static Knobs k = knobs_from_env();
  return k;
}

const DeviceInfo& device_info() {
  static const DeviceInfo unknown;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return unknown;
  std::lock_guard<std::mutex> lk(g_dev_mu);
  if (!g_dev_known[dev]) {
    DeviceInfo d;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) d.cus = cus;
    const int x = query_xcds(dev);
    if (x >= 1 && x <= kMaxXcds) d.xcds = x;
    g_dev[dev] = d;
    g_dev_known[dev] = true;
  }
  return g_dev[dev];
}

}  // namespace st

extern "C" int st_testing_set(const char* name, double value) {
  if (name == nullptr) return 1;
  st::Knobs& k = st::knobs();
  const int v = (int)value;
  if (!strcmp(name, "fwd_fast")) k.fwd_fast = v;
  else if (!strcmp(name, "dq_fast")) k.dq_fast = v;
  else if (!strcmp(name, "dkv_fast")) k.dkv_fast = v;
  else if (!strcmp(name, "dkv_queue")) k.dkv_queue = v;
  else if (!strcmp(name, "fwd_wq") && (v == 32 || v == 64)) k.fwd_wq = v;
  else if (!strcmp(name, "fwd_pipe")) k.fwd_pipe = v;
  else if (!strcmp(name, "fwd_gap") && value >= 0.0 && value <= 64.0) k.fwd_gap = (float)value;
  else return 1;
  return 0;
}

extern "C" int st_testing_device(int* cus, int* xcds) {
  const st::DeviceInfo& d = st::device_info();
  if (cus) *cus = d.cus;
  if (xcds) *xcds = d.xcds;
  return d.cus > 0 ? 0 : 1;
}
