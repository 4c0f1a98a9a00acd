// Host-side plan: graph + schedule -> validated event list, launch list, arena layout.
// Follows the paper's Algorithm 1 / Algorithm 2 symbolically; no device work here.
#pragma once
#include <cstdint>
#include <map>
#include <set>
#include <stdexcept>
#include <string>
#include <vector>

#include "../../include/monet.h"

namespace monet {

constexpr int64_t kAlign = 256;
inline int64_t align_up(int64_t b) { return (b + kAlign - 1) / kAlign * kAlign; }

struct PlanError : std::runtime_error {
    int code;
    PlanError(int c, const std::string &m) : std::runtime_error(m), code(c) {}
};

using Attrs = std::map<std::string, std::string>;

struct FwdImpl {
    std::string algo;
    int64_t ws = 0;
    double cost = 0;
    bool inplace = false;
    Attrs extra;
};
struct BwdImpl {
    std::string algo;
    std::vector<int> deps;
    int64_t ws = 0;
    double cost = 0;
    Attrs extra;
};
struct Node {
    int id = 0;
    std::string op;
    std::vector<int> ins, pars;
    std::vector<int64_t> shape;
    Attrs attrs;
    std::vector<FwdImpl> fimpls;
    bool aux = false, persist = false;
    int64_t bytes = 0;            // |x_i|: logical bytes (0 for persistent nodes)
    std::vector<int> consumers;   // real operators reading this output
    std::vector<int> aux_children;
    int attr_int(const char *k, int dflt = 0) const;
    double attr_f(const char *k, double dflt = 0) const;
};
struct Ext {
    std::string name, dtype;
    std::vector<int64_t> shape;
};
struct Param {
    std::string name;
    std::vector<int64_t> shape;
};
struct Bop {
    int k = 0;
    std::string kind;
    int node = 0;
    std::vector<BwdImpl> impls;
};

struct Graph {
    std::vector<Ext> exts;      // index = -ref
    std::vector<Param> params;  // index = pid
    std::vector<Node> nodes;    // index = id (0 unused)
    std::vector<Bop> bops;      // index = k (0 unused)
    int N() const { return (int)nodes.size() - 1; }
    int B() const { return (int)bops.size() - 1; }
    const std::vector<int64_t> &shape_of(int ref) const { return ref <= 0 ? exts[-ref].shape : nodes[ref].shape; }
    void parse(const std::string &text);
};

struct Schedule {
    std::vector<int> fwd_impl;                // per node
    std::vector<char> fwd_save;               // s^N
    std::vector<int> stage_impl;              // per backward operator
    std::vector<std::map<int, int>> r;        // r[k][i] = implementation
    std::vector<std::set<int>> s;             // s[k] = { i : s^{k-1}_i = 1 }
    void parse(const std::string &text, const Graph &g);
    const std::set<int> &entering(int k, int B, const std::set<int> &fwd) const { return k == B ? fwd : s[k + 1]; }
};

// where a kernel argument lives
enum Region { R_NONE = 0, R_ARENA, R_EXT, R_PARAM, R_PGRAD, R_PERSIST };
struct Ref {
    int region = R_NONE;
    int64_t off = 0;   // byte offset (arena / persist) or index (ext / param / pgrad)
};

struct Launch {
    size_t event = 0;      // index of the RUN_* record in the trace
    int kind = 0;          // EV_RUN_FWD / RECOMPUTE / BWD
    int id = 0;            // node id or backward operator k
    int impl = 0;
    uint32_t flags = 0;    // same as the record's aux field
    // forward:  a[0], a[1] inputs; a[2] output; a[3] intermediate (mask / index); a[4] workspace
    // backward: a[0] incoming gradient; a[1] forward dependency; a[2], a[3] gradient outputs
    //           for input 0 / 1; a[4] workspace
    Ref a[5];
};

struct PoisonFill {
    size_t before_launch;  // fill happens before this launch index (== launches.size() -> at end)
    int64_t off, bytes;
};

enum { EV_ALLOC = 0, EV_FREE, EV_RUN_FWD, EV_RUN_RECOMPUTE, EV_RUN_BWD, EV_SAVE, EV_ALIAS };
enum { T_FWD = 0, T_GRAD, T_FWS, T_BWS };

struct Plan {
    Graph g;
    Schedule sch;
    std::vector<monet_event> events;
    std::vector<Launch> launches;
    std::vector<PoisonFill> poison;
    // (event index, node, is_grad) -> offset, for tests that read tensors back
    std::vector<std::map<std::pair<int, int>, int64_t>> where;   // per launch: live tensor offsets
    std::map<int, int64_t> bn_stats_off;   // node -> offset in the persistent region
    int64_t loss_off = 0;
    int64_t scratch_off = 0, scratch_bytes = 0;
    int64_t persistent_bytes = 0;
    int64_t dynamic_bytes = 0;   // physical high-water mark of the arena
    int64_t exact_peak = 0, predicted_peak = 0, predicted_peak_tight = 0;

    void build(const std::string &graph_text, const std::string &schedule_text);

  private:
    void validate() const;
    void lower();
    void closed_form();
};

}  // namespace monet
