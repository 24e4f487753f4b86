// Error text and the per-kernel timing bracket.
#include "common.h"

#include <cstring>
#include <string>
#include <vector>

namespace gnn {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
void clear_error() { g_err[0] = 0; }

// ---- tuning knobs -------------------------------------------------------------
// block_cols: gathered vertices per column block of the blocked edge lists.  A block
// of 128-byte row slices (one slice per XCD) should sit in one XCD's 4 MB L2:
// 24576 * 128 B = 3 MB (the measured optimum at the Reddit-scale workload; fewer,
// larger blocks save accumulator read-modify-writes, more would spill the L2).
// 0 disables blocking.
static int64_t g_config[kCfgCount] = {24576, 0};
int64_t config_get(ConfigKey k) { return g_config[k]; }

// ---- profiling ---------------------------------------------------------------
struct Pending {
  const char* name;
  hipEvent_t a, b;
};
struct Total {
  const char* name;
  double ms;
  int64_t launches;
};
static bool g_prof_on = false;
static std::vector<Pending> g_pending;
static std::vector<Total> g_totals;
static std::vector<hipEvent_t> g_free_events;
static Pending g_open;

static hipEvent_t get_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

void prof_begin(const char* name, hipStream_t s) {
  if (!g_prof_on) return;
  g_open.name = name;
  g_open.a = get_event();
  g_open.b = get_event();
  (void)hipEventRecord(g_open.a, s);
}

void prof_end(hipStream_t s) {
  if (!g_prof_on) return;
  (void)hipEventRecord(g_open.b, s);
  g_pending.push_back(g_open);
}

}  // namespace gnn

using namespace gnn;

extern "C" const char* gnn_last_error(void) { return g_err; }

extern "C" gnn_status_t gnn_config_set(const char* key, int64_t value) {
  clear_error();
  GNN_REQUIRE(key != nullptr, GNN_ERR_INVALID_ARG, "gnn_config_set: key is null");
  if (std::strcmp(key, "block_cols") == 0) {
    GNN_REQUIRE(value >= 0 && value <= (1 << 30), GNN_ERR_INVALID_ARG,
                "gnn_config_set: block_cols out of range");
    g_config[kCfgBlockCols] = value;
    return GNN_OK;
  }
  if (std::strcmp(key, "force_simple_kernels") == 0) {
    g_config[kCfgForceSimple] = value != 0;
    return GNN_OK;
  }
  set_error("gnn_config_set: unknown key '%s'", key);
  return GNN_ERR_INVALID_ARG;
}

extern "C" gnn_status_t gnn_prof_enable(int on) {
  g_prof_on = on != 0;
  return GNN_OK;
}

extern "C" gnn_status_t gnn_prof_collect(void) {
  for (Pending& p : g_pending) {
    GNN_HIP(hipEventSynchronize(p.b));
    float ms = 0.f;
    GNN_HIP(hipEventElapsedTime(&ms, p.a, p.b));
    Total* t = nullptr;
    for (Total& c : g_totals)
      if (c.name == p.name || std::strcmp(c.name, p.name) == 0) {
        t = &c;
        break;
      }
    if (!t) {
      g_totals.push_back(Total{p.name, 0.0, 0});
      t = &g_totals.back();
    }
    t->ms += ms;
    t->launches += 1;
    g_free_events.push_back(p.a);
    g_free_events.push_back(p.b);
  }
  g_pending.clear();
  return GNN_OK;
}

extern "C" gnn_status_t gnn_prof_reset(void) {
  GNN_TRY(gnn_prof_collect());
  g_totals.clear();
  return GNN_OK;
}

extern "C" int gnn_prof_count(void) { return static_cast<int>(g_totals.size()); }

extern "C" gnn_status_t gnn_prof_get(int i, const char** name, double* total_ms, int64_t* launches) {
  GNN_REQUIRE(i >= 0 && i < static_cast<int>(g_totals.size()), GNN_ERR_INVALID_ARG,
              "gnn_prof_get: index %d out of range", i);
  if (name) *name = g_totals[i].name;
  if (total_ms) *total_ms = g_totals[i].ms;
  if (launches) *launches = g_totals[i].launches;
  return GNN_OK;
}
