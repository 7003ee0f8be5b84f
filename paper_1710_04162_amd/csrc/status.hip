// Version, status strings and the host-side split rule.
#include "common.h"

extern "C" int synk_version(void) { return SYNK_VERSION; }

extern "C" const char* synk_status_string(int status) {
  switch (status) {
    case SYNK_OK: return "ok";
    case SYNK_ERR_NULL: return "a required pointer is NULL";
    case SYNK_ERR_SHAPE: return "a size or count is out of range or inconsistent";
    case SYNK_ERR_DTYPE: return "element type not supported by this call";
    case SYNK_ERR_OP: return "reduce op unknown or not defined for the element type";
    case SYNK_ERR_ALIGN: return "a device pointer is not aligned as documented";
    case SYNK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SYNK_ERR_INDEX: return "an index was out of range";
    case SYNK_ERR_HIP: return "a HIP runtime call failed";
    case SYNK_ERR_UNSUPPORTED: return "request outside what is implemented";
    default: return "unknown status";
  }
}

// Sec. 3.2 step 1 / Sec. 5.1: contiguous, as equal as possible, remainder to
// the first shares.
extern "C" int synk_split(int64_t count, int parts, int64_t* start) {
  if (!start) return SYNK_ERR_NULL;
  if (count < 0 || parts <= 0) return SYNK_ERR_SHAPE;
  for (int i = 0; i < parts; ++i) {
    int64_t s, n;
    synk::share(count, parts, i, &s, &n);
    start[i] = s;
  }
  start[parts] = count;
  return SYNK_OK;
}

// ---------------------------------------------------------------- profiling
namespace synk {
static thread_local hipEvent_t tl_start = nullptr, tl_stop = nullptr;
static thread_local int tl_kernel = SYNK_KERNEL_MAIN;

static thread_local int tl_held = 0;   // > 0: launches of a nested call leave the pending pair alone

ProfileHold::ProfileHold() { ++tl_held; }
ProfileHold::~ProfileHold() { --tl_held; }

bool take_profile_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop) {
  if (!tl_start || kernel_id != tl_kernel || tl_held > 0) return false;
  *start = tl_start;
  *stop = tl_stop;
  tl_start = tl_stop = nullptr;
  return true;
}
}  // namespace synk

extern "C" int synk_profile_next_launch_of(int kernel, void* start_event, void* stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr)) return SYNK_ERR_NULL;
  if (kernel < 0) return SYNK_ERR_SHAPE;
  synk::tl_start = reinterpret_cast<hipEvent_t>(start_event);
  synk::tl_stop = reinterpret_cast<hipEvent_t>(stop_event);
  synk::tl_kernel = kernel;
  return SYNK_OK;
}

extern "C" int synk_profile_pending(void) { return synk::tl_start != nullptr ? 1 : 0; }

extern "C" int synk_profile_next_launch(void* start_event, void* stop_event) {
  return synk_profile_next_launch_of(SYNK_KERNEL_MAIN, start_event, stop_event);
}
