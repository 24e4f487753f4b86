// Error text and the per-kernel timing bracket.
#include "common.h"

#include <atomic>
#include <cstring>
#include <mutex>
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
// 20480 * 128 B = 2.5 MB (the measured optimum at the Reddit-scale workload once sparse
// blocks share launches; wider blocks spill the L2, narrower ones pay the accumulator
// read-modify-writes more often).
// 0 disables blocking.
// lds_scalar_table: 1 lets the blocked destination-side kernels keep a block's el table in LDS
// gcn_mapping: thread mapping of the GCN aggregation, 0 vertex-balanced, 1 edge-balanced,
// 2 (default) per graph what gnn_gcn_tune measured, vertex-balanced where it never ran
// gmm_mapping: the same for the forward aggregation of the GMM layer (gnn_gmm_tune)
// blocked_min_edges: mean edges per (row, column block) from which the column-blocked kernels are
// used (below that the per-launch cost of visiting every row outweighs the cache residency;
// break-even measured between 12 and 24 at 1 KB rows)
// gather_precision: 0 the column-blocked GAT kernels gather fp32 rows, 1 they gather an fp16 copy
// merge_blocks: 1 (default) adjacent sparse column blocks share one launch of a blocked kernel
// (read at gnn_graph_create), 0 every block has its own launch
// wide_offsets: 1 makes the column-blocked GAT kernels address gathered rows with 64-bit offsets
// also where 32 bits reach every row (the path of matrices of 4 GB and more; a test hook)
// resident_sums: 1 (default) lets the column-blocked aggregations run all blocks in one persistent
// launch that keeps the rows' running sums on the chip (LDS); 0: one launch per block or group of
// blocks, the sums read and written in between
static std::atomic<int64_t> g_config[kCfgCount] = {{12288}, {0}, {1}, {2}, {2}, {16}, {0}, {1}, {0}, {1}, {4096}, {0}};
// resident_sync_every: the workgroups of an XCD meet after every k-th column block (0, default: once
// per generation of rows, after the last block)
// resident_spin: polls after which a workgroup of that launch stops waiting for the others of its XCD
// at a block boundary (the wait only paces the workgroups; 0 = never wait)
int64_t config_get(ConfigKey k) { return g_config[k].load(std::memory_order_relaxed); }

static int query_cu_count() {
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
    return v;
  return 256;
}
int device_cu_count() {
  static const int cus = query_cu_count();  // one GPU type per process; initialised once, thread-safe
  return cus;
}

// ---- profiling ---------------------------------------------------------------
struct Pending {
  const char* name;
  hipEvent_t a, b;
  bool closed = false;
};
struct Total {
  const char* name;
  double ms;
  int64_t launches;
};
static std::atomic<bool> g_prof_on{false};
static std::mutex g_prof_mu;  // guards everything below
static std::vector<Pending> g_pending;
static std::vector<Total> g_totals;
static std::vector<hipEvent_t> g_free_events;
static int64_t g_generation = 0;  // bumped whenever g_pending is emptied: stale slots are ignored
constexpr int64_t kSlotBits = 32;

static hipEvent_t get_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

int64_t prof_begin(const char* name, hipStream_t s) {
  if (!g_prof_on.load(std::memory_order_relaxed)) return -1;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  Pending p{name, get_event(), get_event()};
  if (!p.a || !p.b) {
    if (p.a) g_free_events.push_back(p.a);
    if (p.b) g_free_events.push_back(p.b);
    return -1;
  }
  (void)hipEventRecord(p.a, s);
  g_pending.push_back(p);
  return (g_generation << kSlotBits) | static_cast<int64_t>(g_pending.size() - 1);
}

void prof_end(int64_t token, hipStream_t s) {
  if (token < 0) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  // gnn_prof_collect may have run in between (it drops unfinished brackets)
  if ((token >> kSlotBits) != g_generation) return;
  const size_t slot = static_cast<size_t>(token & ((int64_t(1) << kSlotBits) - 1));
  if (slot < g_pending.size() && !g_pending[slot].closed) {
    (void)hipEventRecord(g_pending[slot].b, s);
    g_pending[slot].closed = true;
  }
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
    g_config[kCfgBlockCols].store(value);
    return GNN_OK;
  }
  if (std::strcmp(key, "force_simple_kernels") == 0) {
    g_config[kCfgForceSimple].store(value != 0);
    return GNN_OK;
  }
  if (std::strcmp(key, "lds_scalar_table") == 0) {
    g_config[kCfgLdsScalarTable].store(value != 0);
    return GNN_OK;
  }
  if (std::strcmp(key, "gcn_mapping") == 0) {
    GNN_REQUIRE(value >= 0 && value <= 2, GNN_ERR_INVALID_ARG, "gnn_config_set: gcn_mapping must be 0, 1 or 2");
    g_config[kCfgGcnMapping].store(value);
    return GNN_OK;
  }
  if (std::strcmp(key, "gather_precision") == 0) {
    GNN_REQUIRE(value == 0 || value == 1, GNN_ERR_INVALID_ARG, "gnn_config_set: gather_precision must be 0 or 1");
    g_config[kCfgGatherPrecision].store(value);
    return GNN_OK;
  }
  if (std::strcmp(key, "wide_offsets") == 0) {
    g_config[kCfgWideOffsets].store(value != 0);
    return GNN_OK;
  }
  if (std::strcmp(key, "resident_sums") == 0) {
    g_config[kCfgResidentSums].store(value != 0);
    return GNN_OK;
  }
  if (std::strcmp(key, "resident_sync_every") == 0) {
    GNN_REQUIRE(value >= 0 && value <= 64, GNN_ERR_INVALID_ARG, "gnn_config_set: resident_sync_every must be 0 .. 64");
    g_config[kCfgResidentSyncEvery].store(value);
    return GNN_OK;
  }
  if (std::strcmp(key, "resident_spin") == 0) {
    GNN_REQUIRE(value >= 0 && value <= (1 << 24), GNN_ERR_INVALID_ARG, "gnn_config_set: resident_spin out of range");
    g_config[kCfgResidentSpin].store(value);
    return GNN_OK;
  }
  if (std::strcmp(key, "merge_blocks") == 0) {
    g_config[kCfgMergeBlocks].store(value != 0);
    return GNN_OK;
  }
  if (std::strcmp(key, "blocked_min_edges") == 0) {
    GNN_REQUIRE(value >= 0 && value <= (1 << 20), GNN_ERR_INVALID_ARG,
                "gnn_config_set: blocked_min_edges out of range");
    g_config[kCfgBlockedMinEdges].store(value);
    return GNN_OK;
  }
  if (std::strcmp(key, "gmm_mapping") == 0) {
    GNN_REQUIRE(value >= 0 && value <= 2, GNN_ERR_INVALID_ARG, "gnn_config_set: gmm_mapping must be 0, 1 or 2");
    g_config[kCfgGmmMapping].store(value);
    return GNN_OK;
  }
  set_error("gnn_config_set: unknown key '%s'", key);
  return GNN_ERR_INVALID_ARG;
}

extern "C" gnn_status_t gnn_prof_enable(int on) {
  g_prof_on.store(on != 0);
  return GNN_OK;
}

static gnn_status_t collect_locked() {
  for (Pending& p : g_pending) {
    if (!p.closed) {  // a bracket still open on another thread: drop it
      g_free_events.push_back(p.a);
      g_free_events.push_back(p.b);
      continue;
    }
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
  ++g_generation;
  return GNN_OK;
}

extern "C" gnn_status_t gnn_prof_collect(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  return collect_locked();
}

extern "C" gnn_status_t gnn_prof_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  GNN_TRY(collect_locked());
  g_totals.clear();
  return GNN_OK;
}

extern "C" int gnn_prof_count(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  return static_cast<int>(g_totals.size());
}

extern "C" gnn_status_t gnn_prof_get(int i, const char** name, double* total_ms, int64_t* launches) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  GNN_REQUIRE(i >= 0 && i < static_cast<int>(g_totals.size()), GNN_ERR_INVALID_ARG,
              "gnn_prof_get: index %d out of range", i);
  if (name) *name = g_totals[i].name;
  if (total_ms) *total_ms = g_totals[i].ms;
  if (launches) *launches = g_totals[i].launches;
  return GNN_OK;
}
