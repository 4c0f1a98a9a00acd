// Plan construction: text -> graph/schedule -> feasibility checks -> symbolic run of the
// forward pass (Algorithm 1) and the backward pass with recomputation (Algorithm 2)
// -> event trace, kernel launch list with resolved arena offsets, predicted peak.
#include "plan.hpp"

#include <algorithm>
#include <deque>
#include <sstream>

namespace monet {

// ------------------------------------------------------------------ small helpers
static std::vector<std::string> split_ws(const std::string &line) {
    std::vector<std::string> out;
    std::istringstream is(line);
    std::string tok;
    while (is >> tok) out.push_back(tok);
    return out;
}
static std::vector<int64_t> parse_dims(const std::string &s) {
    std::vector<int64_t> d;
    size_t p = 0;
    while (p <= s.size()) {
        size_t q = s.find('x', p);
        if (q == std::string::npos) q = s.size();
        d.push_back(std::stoll(s.substr(p, q - p)));
        p = q + 1;
    }
    return d;
}
static std::vector<int> parse_refs(const std::string &s) {
    std::vector<int> r;
    if (s == "-") return r;
    size_t p = 0;
    while (p <= s.size()) {
        size_t q = s.find(',', p);
        if (q == std::string::npos) q = s.size();
        r.push_back(std::stoi(s.substr(p, q - p)));
        p = q + 1;
    }
    return r;
}
static Attrs parse_kv(const std::vector<std::string> &f, size_t from) {
    Attrs a;
    for (size_t i = from; i < f.size(); ++i) {
        size_t e = f[i].find('=');
        if (e == std::string::npos) throw PlanError(MONET_BAD_GRAPH, "field without '=': " + f[i]);
        a[f[i].substr(0, e)] = f[i].substr(e + 1);
    }
    return a;
}
static std::string take(Attrs &a, const char *k) {
    auto it = a.find(k);
    if (it == a.end()) throw PlanError(MONET_BAD_GRAPH, std::string("missing field ") + k);
    std::string v = it->second;
    a.erase(it);
    return v;
}
static int64_t numel(const std::vector<int64_t> &s) {
    int64_t n = 1;
    for (auto d : s) n *= d;
    return n;
}
static std::vector<std::string> lines_of(const std::string &text) {
    std::vector<std::string> out;
    std::istringstream is(text);
    std::string ln;
    while (std::getline(is, ln)) {
        size_t h = ln.find('#');
        if (h != std::string::npos) ln.resize(h);
        if (!split_ws(ln).empty()) out.push_back(ln);
    }
    return out;
}

int Node::attr_int(const char *k, int dflt) const {
    auto it = attrs.find(k);
    return it == attrs.end() ? dflt : std::stoi(it->second);
}
double Node::attr_f(const char *k, double dflt) const {
    auto it = attrs.find(k);
    return it == attrs.end() ? dflt : std::stod(it->second);
}

// ------------------------------------------------------------------ parsing
void Graph::parse(const std::string &text) {
    auto lines = lines_of(text);
    if (lines.empty() || split_ws(lines[0]) != std::vector<std::string>{"monet-graph", "1"})
        throw PlanError(MONET_BAD_GRAPH, "graph text must start with 'monet-graph 1'");
    nodes.assign(1, Node());
    bops.assign(1, Bop());
    try {
        for (size_t li = 1; li < lines.size(); ++li) {
            auto f = split_ws(lines[li]);
            const std::string &tag = f[0];
            if (tag == "ext") {
                int ref = std::stoi(f.at(1));
                if (-ref != (int)exts.size()) throw PlanError(MONET_BAD_GRAPH, "ext records must be numbered 0,-1,...");
                exts.push_back(Ext{f.at(2), f.at(3), parse_dims(f.at(4))});
            } else if (tag == "param") {
                if (std::stoi(f.at(1)) != (int)params.size()) throw PlanError(MONET_BAD_GRAPH, "param records must be numbered 0,1,...");
                params.push_back(Param{f.at(2), parse_dims(f.at(3))});
            } else if (tag == "node") {
                Node n;
                n.id = std::stoi(f.at(1));
                if (n.id != (int)nodes.size()) throw PlanError(MONET_BAD_GRAPH, "node records must be numbered 1,2,...");
                n.op = f.at(2);
                Attrs a = parse_kv(f, 3);
                n.ins = parse_refs(take(a, "in"));
                n.pars = parse_refs(take(a, "par"));
                n.shape = parse_dims(take(a, "shape"));
                n.attrs = a;
                n.aux = (n.op == "mask" || n.op == "poolidx");
                n.persist = n.attr_int("persist") == 1;
                int64_t esz = n.op == "mask" ? 8 : (n.op == "poolidx" ? 1 : 4);
                n.bytes = n.persist ? 0 : align_up(numel(n.shape) * esz);
                for (int j : n.ins)
                    if (j >= n.id || -j >= (int)exts.size())
                        throw PlanError(MONET_BAD_GRAPH, "node " + std::to_string(n.id) + ": input " + std::to_string(j) + " does not precede it");
                for (int p : n.pars)
                    if (p < 0 || p >= (int)params.size()) throw PlanError(MONET_BAD_GRAPH, "node " + std::to_string(n.id) + ": unknown parameter");
                nodes.push_back(n);
            } else if (tag == "fimpl") {
                int i = std::stoi(f.at(1)), l = std::stoi(f.at(2));
                if (i < 1 || i >= (int)nodes.size() || l != (int)nodes[i].fimpls.size())
                    throw PlanError(MONET_BAD_GRAPH, "fimpl records out of order at node " + std::to_string(i));
                Attrs a = parse_kv(f, 3);
                FwdImpl im;
                im.algo = take(a, "algo");
                im.ws = std::stoll(take(a, "ws"));
                im.cost = std::stod(take(a, "cost"));
                im.inplace = a.count("inplace") && a["inplace"] == "1";
                im.extra = a;
                nodes[i].fimpls.push_back(im);
            } else if (tag == "bop") {
                Bop b;
                b.k = std::stoi(f.at(1));
                if (b.k != (int)bops.size()) throw PlanError(MONET_BAD_GRAPH, "bop records must be numbered 1,2,...");
                b.kind = f.at(2);
                Attrs a = parse_kv(f, 3);
                b.node = std::stoi(take(a, "node"));
                if (b.node < 1 || b.node >= (int)nodes.size()) throw PlanError(MONET_BAD_GRAPH, "bop on unknown node");
                if (b.k > 1 && bops.back().node > b.node) throw PlanError(MONET_BAD_GRAPH, "bop records must follow node order");
                bops.push_back(b);
            } else if (tag == "bimpl") {
                int k = std::stoi(f.at(1)), l = std::stoi(f.at(2));
                if (k < 1 || k >= (int)bops.size() || l != (int)bops[k].impls.size())
                    throw PlanError(MONET_BAD_GRAPH, "bimpl records out of order at operator " + std::to_string(k));
                Attrs a = parse_kv(f, 3);
                BwdImpl im;
                im.algo = take(a, "algo");
                im.deps = parse_refs(take(a, "deps"));
                im.ws = std::stoll(take(a, "ws"));
                im.cost = std::stod(take(a, "cost"));
                im.extra = a;
                bops[k].impls.push_back(im);
            } else {
                throw PlanError(MONET_BAD_GRAPH, "unknown record '" + tag + "'");
            }
        }
    } catch (const PlanError &) {
        throw;
    } catch (const std::exception &e) {
        throw PlanError(MONET_BAD_GRAPH, std::string("malformed graph text: ") + e.what());
    }
    for (auto &n : nodes) {
        if (n.id == 0) continue;
        if (n.aux) {
            if (n.ins.size() != 1 || n.ins[0] != n.id - 1 || nodes[n.ins[0]].aux)
                throw PlanError(MONET_BAD_GRAPH, "aux node " + std::to_string(n.id) + " must directly follow its creator");
            nodes[n.ins[0]].aux_children.push_back(n.id);
        } else {
            if (n.fimpls.empty()) throw PlanError(MONET_BAD_GRAPH, "node " + std::to_string(n.id) + " has no forward implementation");
            for (int j : n.ins)
                if (j > 0) {
                    if (nodes[j].aux || nodes[j].persist)
                        throw PlanError(MONET_BAD_GRAPH, "node " + std::to_string(n.id) + " reads an aux or persistent node");
                    nodes[j].consumers.push_back(n.id);
                }
        }
    }
    for (auto &b : bops)
        if (b.k && b.impls.empty()) throw PlanError(MONET_BAD_GRAPH, "backward operator " + std::to_string(b.k) + " has no implementation");
}

void Schedule::parse(const std::string &text, const Graph &g) {
    auto lines = lines_of(text);
    if (lines.empty() || split_ws(lines[0]) != std::vector<std::string>{"monet-schedule", "1"})
        throw PlanError(MONET_BAD_GRAPH, "schedule text must start with 'monet-schedule 1'");
    const int N = g.N(), B = g.B();
    fwd_impl.assign(N + 1, -2);
    fwd_save.assign(N + 1, 0);
    stage_impl.assign(B + 1, -2);
    r.assign(B + 2, {});
    s.assign(B + 2, {});
    try {
        for (size_t li = 1; li < lines.size(); ++li) {
            auto f = split_ws(lines[li]);
            if (f[0] == "fwd") {
                int i = std::stoi(f.at(1));
                Attrs a = parse_kv(f, 2);
                if (i < 1 || i > N) throw PlanError(MONET_BAD_GRAPH, "fwd record for unknown node");
                fwd_impl[i] = std::stoi(take(a, "impl"));
                fwd_save[i] = take(a, "save") == "1";
            } else if (f[0] == "stage") {
                int k = std::stoi(f.at(1));
                Attrs a = parse_kv(f, 2);
                if (k < 1 || k > B) throw PlanError(MONET_BAD_GRAPH, "stage record for unknown backward operator");
                stage_impl[k] = std::stoi(take(a, "impl"));
            } else if (f[0] == "r") {
                int k = std::stoi(f.at(1)), i = std::stoi(f.at(2));
                Attrs a = parse_kv(f, 3);
                if (k < 1 || k > B || i < 1 || i > N) throw PlanError(MONET_BAD_GRAPH, "r record out of range");
                r[k][i] = std::stoi(take(a, "impl"));
            } else if (f[0] == "s") {
                int k = std::stoi(f.at(1)), i = std::stoi(f.at(2));
                if (k < 1 || k > B || i < 1 || i > N) throw PlanError(MONET_BAD_GRAPH, "s record out of range");
                s[k].insert(i);
            } else {
                throw PlanError(MONET_BAD_GRAPH, "unknown schedule record '" + f[0] + "'");
            }
        }
    } catch (const PlanError &) {
        throw;
    } catch (const std::exception &e) {
        throw PlanError(MONET_BAD_GRAPH, std::string("malformed schedule text: ") + e.what());
    }
    for (int i = 1; i <= N; ++i)
        if (fwd_impl[i] == -2) throw PlanError(MONET_BAD_GRAPH, "schedule has no fwd record for node " + std::to_string(i));
    for (int k = 1; k <= B; ++k)
        if (stage_impl[k] == -2) throw PlanError(MONET_BAD_GRAPH, "schedule has no stage record for operator " + std::to_string(k));
}

// ------------------------------------------------------------------ what each backward implementation reads
static std::vector<int> node_deps(const Graph &g, int k, int l) {
    std::vector<int> d;
    for (int j : g.bops[k].impls[l].deps)
        if (j > 0) d.push_back(j);
    return d;
}

// The dependency sets D_k^l are part of the graph text; the kernels below them are fixed,
// so the text must agree with what each kernel actually reads.
static void check_declared_deps(const Graph &g) {
    for (int k = 1; k <= g.B(); ++k) {
        const Bop &b = g.bops[k];
        const Node &n = g.nodes[b.node];
        for (size_t l = 0; l < b.impls.size(); ++l) {
            const std::string &algo = b.impls[l].algo;
            std::vector<int> want;
            bool known = true;
            auto input0 = [&] { if (n.ins[0] > 0) want.push_back(n.ins[0]); };
            auto aux0 = [&] {
                if (n.aux_children.empty()) throw PlanError(MONET_BAD_GRAPH, "node " + std::to_string(n.id) + " has no intermediate node");
                want.push_back(n.aux_children[0]);
            };
            if (b.kind == "conv_wgrad") { known = (algo == "direct" || algo == "splitk" || algo == "winograd" || algo == "winograd4" || algo == "im2col"); input0(); }
            else if (b.kind == "conv_dgrad") { known = (algo == "igemm" || algo == "igemm_splitk" || algo == "winograd" || algo == "winograd4" || algo == "winograd4f"); }
            else if (b.kind == "tconv_wgrad") { known = (algo == "direct" || algo == "splitk"); input0(); }
            else if (b.kind == "tconv_dgrad") { known = algo == "igemm"; }
            else if (b.kind == "dwconv_wgrad") { known = algo == "direct"; input0(); }
            else if (b.kind == "dwconv_dgrad") { known = algo == "direct"; }
            else if (b.kind == "concat_bwd") { known = algo == "copy"; }
            else if (b.kind == "linear_wgrad") { known = algo == "gemm"; input0(); }
            else if (b.kind == "linear_dgrad") { known = algo == "gemm"; }
            else if (b.kind == "bn_bwd") {
                if (algo == "from_input") input0(); else if (algo == "from_output") want.push_back(n.id); else known = false;
            } else if (b.kind == "relu_bwd" || b.kind == "relu6_bwd") {
                if (algo == "from_input") input0(); else if (algo == "from_output") want.push_back(n.id);
                else if (algo == "from_mask") aux0(); else known = false;
            } else if (b.kind == "maxpool_bwd") {
                if (algo == "from_input") input0(); else if (algo == "from_index") aux0(); else known = false;
            } else if (b.kind == "add_bwd") { known = algo == "copy"; }
            else if (b.kind == "avgpool_bwd") { known = algo == "direct"; }
            else if (b.kind == "softmaxce_bwd") { known = algo == "direct"; input0(); }
            else if (b.kind == "sumloss_bwd") { known = algo == "fill"; }
            else throw PlanError(MONET_BAD_GRAPH, "unknown backward operator kind " + b.kind);
            if (!known) throw PlanError(MONET_BAD_GRAPH, "backward operator " + std::to_string(k) + ": unknown implementation " + algo);
            if (node_deps(g, k, (int)l) != want)
                throw PlanError(MONET_BAD_GRAPH, "backward operator " + std::to_string(k) + " (" + algo + "): declared dependencies differ from what the kernel reads");
        }
    }
}

static std::vector<int> grad_positions(const Graph &g, const Bop &b) {
    std::vector<int> p;
    const std::string &kd = b.kind;
    if (kd.size() > 6 && kd.compare(kd.size() - 6, 6, "_wgrad") == 0) return p;
    const Node &n = g.nodes[b.node];
    if (kd == "softmaxce_bwd") { p.push_back(0); return p; }
    for (size_t i = 0; i < n.ins.size(); ++i)
        if (n.ins[i] > 0) p.push_back((int)i);
    return p;
}

// ------------------------------------------------------------------ feasibility (Eq. 7, Eq. 8, Appendix C.3 / D)
void Plan::validate() const {
    const int N = g.N(), B = g.B();
    auto S = [](int v) { return std::to_string(v); };
    std::set<int> fsave;
    for (int i = 1; i <= N; ++i) {
        const Node &n = g.nodes[i];
        int l = sch.fwd_impl[i];
        if (n.aux) {
            if (l != -1) throw PlanError(MONET_INFEASIBLE, "aux node " + S(i) + " carries a forward implementation");
        } else if (l < 0 || l >= (int)n.fimpls.size()) {
            throw PlanError(MONET_INFEASIBLE, "delta: node " + S(i) + " has no forward implementation " + S(l));
        }
        if (sch.fwd_save[i]) {
            if (n.persist) throw PlanError(MONET_INFEASIBLE, "node " + S(i) + " is persistent and cannot be saved");
            fsave.insert(i);
        }
    }
    for (int k = 1; k <= B; ++k)
        if (sch.stage_impl[k] < 0 || sch.stage_impl[k] >= (int)g.bops[k].impls.size())
            throw PlanError(MONET_INFEASIBLE, "delta-hat: backward operator " + S(k) + " has no implementation " + S(sch.stage_impl[k]));
    auto inplace_shape_ok = [&](const Node &n) {
        int j = n.ins[0];
        return j > 0 && !g.nodes[j].aux && g.nodes[j].bytes == n.bytes;
    };
    for (int i = 1; i <= N; ++i) {
        const Node &n = g.nodes[i];
        if (n.aux || !n.fimpls[sch.fwd_impl[i]].inplace) continue;
        if (!inplace_shape_ok(n)) throw PlanError(MONET_INFEASIBLE, "C.3: node " + S(i) + " cannot run in place over its input");
        int j = n.ins[0];
        if (sch.fwd_save[j]) throw PlanError(MONET_INFEASIBLE, "C.3: node " + S(i) + " runs in place over " + S(j) + ", which the forward pass saves");
        for (int t : g.nodes[j].consumers)
            if (t != i) throw PlanError(MONET_INFEASIBLE, "C.3: node " + S(i) + " runs in place over " + S(j) + ", which another operator reads");
    }
    for (int k = B; k >= 1; --k) {
        const auto &rk = sch.r[k];
        const auto &sk = sch.s[k];
        const auto &enter = sch.entering(k, B, fsave);
        const int fk = g.bops[k].node;
        std::vector<int> D = node_deps(g, k, sch.stage_impl[k]);
        std::map<int, int> overwritten;
        for (auto &kv : rk) {
            int i = kv.first, l = kv.second;
            const Node &n = g.nodes[i];
            std::string at = "stage " + S(k) + ": ";
            if (enter.count(i)) throw PlanError(MONET_INFEASIBLE, at + "node " + S(i) + " is recomputed although it is already held");
            if (i > fk && !(n.aux && n.ins[0] == fk))
                throw PlanError(MONET_INFEASIBLE, "Appendix B: stage " + S(k) + " recomputes node " + S(i) + " beyond its own node " + S(fk));
            if (n.persist) throw PlanError(MONET_INFEASIBLE, at + "persistent node " + S(i) + " cannot be recomputed");
            if (n.aux) {
                if (l != -1 || !rk.count(n.ins[0]))
                    throw PlanError(MONET_INFEASIBLE, "Appendix D: aux node " + S(i) + " recomputed at stage " + S(k) + " without its creator");
                continue;
            }
            if (l < 0 || l >= (int)n.fimpls.size()) throw PlanError(MONET_INFEASIBLE, "delta^k: node " + S(i) + " has no forward implementation " + S(l));
            for (int j : n.ins) {
                if (j <= 0) continue;
                if (overwritten.count(j))
                    throw PlanError(MONET_INFEASIBLE, "C.3: stage " + S(k) + " node " + S(i) + " reads " + S(j) + ", overwritten in place by " + S(overwritten[j]));
                if (!sk.count(j) && !rk.count(j))
                    throw PlanError(MONET_INFEASIBLE, "Eq.7: stage " + S(k) + " recomputes node " + S(i) + " but input " + S(j) + " is neither saved nor recomputed");
            }
            if (n.fimpls[l].inplace) {
                int j = n.ins[0];
                if (!inplace_shape_ok(n) || !rk.count(j)) throw PlanError(MONET_INFEASIBLE, "C.3: stage " + S(k) + " node " + S(i) + " cannot run in place over its input");
                if (sk.count(j)) throw PlanError(MONET_INFEASIBLE, "C.3: stage " + S(k) + " node " + S(i) + " runs in place over saved tensor " + S(j));
                if (std::find(D.begin(), D.end(), j) != D.end())
                    throw PlanError(MONET_INFEASIBLE, "C.3: stage " + S(k) + " node " + S(i) + " overwrites dependency " + S(j) + " of the backward operator");
                for (int t : g.nodes[j].consumers)
                    if (t > i && rk.count(t))
                        throw PlanError(MONET_INFEASIBLE, "C.3: stage " + S(k) + " node " + S(i) + " overwrites " + S(j) + ", still read by a later recomputation");
                overwritten[j] = i;
            }
        }
        for (int i : sk) {
            if (g.nodes[i].persist) throw PlanError(MONET_INFEASIBLE, "stage " + S(k) + ": persistent node " + S(i) + " cannot be saved");
            if (!enter.count(i) && !rk.count(i))
                throw PlanError(MONET_INFEASIBLE, "Eq.7: stage " + S(k) + " saves node " + S(i) + ", which is neither held nor recomputed");
            if (overwritten.count(i)) throw PlanError(MONET_INFEASIBLE, "C.3: stage " + S(k) + " saves node " + S(i) + ", overwritten in place");
        }
        for (int d : D) {
            if (!sk.count(d) && !rk.count(d))
                throw PlanError(MONET_INFEASIBLE, "Eq.8: backward operator " + S(k) + " depends on node " + S(d) + ", neither saved nor recomputed");
            if (overwritten.count(d)) throw PlanError(MONET_INFEASIBLE, "C.3: backward operator " + S(k) + " depends on node " + S(d) + ", overwritten in place");
        }
    }
}

// ------------------------------------------------------------------ arena: offsets for a known alloc/free sequence
namespace {
struct Arena {
    std::map<int64_t, int64_t> free_;   // offset -> size, coalesced, none touching top
    int64_t top = 0, high = 0;
    int64_t alloc(int64_t sz) {
        auto best = free_.end();
        for (auto it = free_.begin(); it != free_.end(); ++it)
            if (it->second >= sz && (best == free_.end() || it->second < best->second)) best = it;
        if (best != free_.end()) {
            int64_t off = best->first, rest = best->second - sz;
            free_.erase(best);
            if (rest > 0) free_[off + sz] = rest;
            return off;
        }
        int64_t off = top;
        top += sz;
        high = std::max(high, top);
        return off;
    }
    void release(int64_t off, int64_t sz) {
        auto nx = free_.lower_bound(off);
        if (nx != free_.end() && off + sz == nx->first) {
            sz += nx->second;
            nx = free_.erase(nx);
        }
        if (nx != free_.begin()) {
            auto pv = std::prev(nx);
            if (pv->first + pv->second == off) {
                off = pv->first;
                sz += pv->second;
                free_.erase(pv);
            }
        }
        if (off + sz == top) top = off;   // give the tail back
        else free_[off] = sz;
    }
};
}  // namespace

// ------------------------------------------------------------------ symbolic run of Algorithm 1 and Algorithm 2
void Plan::lower() {
    const int N = g.N(), B = g.B();
    events.clear();
    launches.clear();
    poison.clear();
    where.clear();
    Arena arena;
    int64_t live = 0, peak = 0;
    std::map<int, std::pair<int64_t, int64_t>> held;    // forward tensor -> (offset, bytes)
    std::map<int, std::pair<int64_t, int64_t>> grads;   // node -> (offset, bytes) of its gradient

    auto ev = [&](int kind, int stage, int node, int impl, int aux, int64_t bytes) {
        if (kind == EV_ALLOC) live += bytes;
        if (kind == EV_FREE) live -= bytes;
        peak = std::max(peak, live);
        monet_event e{kind, stage, node, impl, aux, 0, bytes, live};
        events.push_back(e);
    };
    // Physical reuse of freed blocks is delayed around bandwidth-bound operators.  The executor may run up to
    // three neighbouring operators of that kind (BatchNorm, add, ReLU and their backward operators) as one
    // kernel; an output of the last must then not sit on memory that an earlier one still reads.  So a block
    // freed right after such a launch goes back to the allocator only once two more launches have been
    // placed, or as soon as a launch of another kind (which ends any such run) is placed; until then only a
    // request of exactly its size may take it.  The events and the
    // live-byte count follow the algorithms exactly; the delay only concerns which offsets later allocations take.
    // The same holds for the small workspace of a recomputed convolution (the cut tiles of the implicit GEMM, the
    // transformed filters of the one-kernel Winograd form): the executor may run the BatchNorm and the ReLU behind it in
    // the convolution's epilogue, whose tiles read the workspace until the last one is done, so the ReLU's buffers must
    // not take its place.  Such a block waits the same way but is never handed to a request of its own size.
    constexpr size_t kReuseLag = 2;
    struct Pending { size_t when; int64_t off, bytes; bool same_size_ok; };
    std::deque<Pending> pending;
    auto chainable = [&](const Launch &L) {
        if (L.kind == EV_RUN_BWD) {
            const std::string &kd = g.bops[L.id].kind;
            return kd == "relu_bwd" || kd == "relu6_bwd" || kd == "add_bwd" || kd == "bn_bwd";
        }
        const std::string &op = g.nodes[L.id].op;
        return op == "bn" || op == "add" || op == "relu" || op == "relu6";
    };
    auto flush_pending = [&](bool all) {
        while (!pending.empty() && (all || pending.front().when + kReuseLag <= launches.size())) {
            arena.release(pending.front().off, pending.front().bytes);
            pending.pop_front();
        }
    };
    // called before the allocations of the launch that is about to be placed
    auto begin_launch = [&](bool is_chainable) { flush_pending(!is_chainable); };
    auto arena_alloc = [&](int stage, int node, int cls, int64_t bytes) {
        flush_pending(false);
        int64_t off = -1;
        // a waiting block of exactly this size may be taken whole: element i of the new tensor then sits on
        // element i of the old one, which the same thread of a fused kernel has read before it writes
        for (auto it = pending.begin(); it != pending.end(); ++it)
            if (it->same_size_ok && it->bytes == bytes) { off = it->off; pending.erase(it); break; }
        if (off < 0) off = arena.alloc(bytes);
        ev(EV_ALLOC, stage, node, -1, cls, bytes);
        return off;
    };
    auto arena_free = [&](int stage, int node, int cls, int64_t off, int64_t bytes) {
        bool conv_ws = false;
        if (cls == T_FWS && !launches.empty() && launches.back().kind == EV_RUN_RECOMPUTE) {
            const Node &n = g.nodes[launches.back().id];
            const std::string &algo = n.fimpls[launches.back().impl].algo;
            conv_ws = n.op == "conv" && algo != "winograd" && algo != "winograd4" && algo != "im2col";
        }
        if (!launches.empty() && chainable(launches.back())) pending.push_back(Pending{launches.size(), off, bytes, true});
        else if (conv_ws) pending.push_back(Pending{launches.size(), off, bytes, false});
        else arena.release(off, bytes);
        ev(EV_FREE, stage, node, -1, cls, bytes);
        poison.push_back(PoisonFill{launches.size(), off, bytes});
    };
    auto fwd_ref = [&](int ref, const std::string &who) {
        Ref r;
        if (ref <= 0) { r.region = R_EXT; r.off = -ref; return r; }
        auto it = held.find(ref);
        if (it == held.end()) throw PlanError(MONET_INFEASIBLE, who + " reads node " + std::to_string(ref) + ", which is not in memory");
        r.region = R_ARENA;
        r.off = it->second.first;
        return r;
    };
    auto snapshot = [&] {
        std::map<std::pair<int, int>, int64_t> m;
        for (auto &h : held) m[{h.first, 0}] = h.second.first;
        for (auto &h : grads) m[{h.first, 1}] = h.second.first;
        where.push_back(m);
    };
    auto run_forward = [&](int i, int l, int stage, const std::vector<int> &emit, int kind) {
        const Node &n = g.nodes[i];
        const FwdImpl &im = n.fimpls[l];
        std::string who = "stage " + std::to_string(stage) + ": node " + std::to_string(i);
        Launch L;
        L.kind = kind; L.id = i; L.impl = l;
        L.flags = (im.inplace ? 1u : 0u) | (emit.empty() ? 0u : 2u);
        begin_launch(chainable(L));
        for (size_t p = 0; p < n.ins.size() && p < 2; ++p) L.a[p] = fwd_ref(n.ins[p], who);
        if (n.persist) { L.a[2].region = R_PERSIST; L.a[2].off = loss_off; }
        else if (im.inplace) L.a[2] = L.a[0];
        else {
            int64_t off = arena_alloc(stage, i, T_FWD, n.bytes);
            held[i] = {off, n.bytes};
            L.a[2].region = R_ARENA; L.a[2].off = off;
        }
        for (int c : emit) {
            int64_t off = arena_alloc(stage, c, T_FWD, g.nodes[c].bytes);
            held[c] = {off, g.nodes[c].bytes};
            L.a[3].region = R_ARENA; L.a[3].off = off;
        }
        int64_t wsb = im.ws > 0 ? align_up(im.ws) : 0, wso = 0;
        if (wsb) { wso = arena_alloc(stage, i, T_FWS, wsb); L.a[4].region = R_ARENA; L.a[4].off = wso; }
        ev(kind, stage, i, l, (int)L.flags, 0);
        L.event = events.size() - 1;
        snapshot();
        launches.push_back(L);
        if (wsb) arena_free(stage, i, T_FWS, wso, wsb);
        if (im.inplace) {
            int j = n.ins[0];
            held[i] = held[j];
            held.erase(j);
            ev(EV_ALIAS, stage, i, -1, j, held[i].second);
        }
    };
    auto drop = [&](int stage, int j) {
        auto h = held[j];
        held.erase(j);
        arena_free(stage, j, T_FWD, h.first, h.second);
    };
    auto ids_upto = [&](int i) {
        std::vector<int> v;
        for (auto &h : held) if (h.first <= i) v.push_back(h.first);
        return v;
    };

    // ---- forward pass
    const int fstage = B + 1;
    for (int i = 1; i <= N; ++i) {
        const Node &n = g.nodes[i];
        if (!n.aux) {
            std::vector<int> emit;
            for (int c : n.aux_children) if (sch.fwd_save[c]) emit.push_back(c);
            run_forward(i, sch.fwd_impl[i], fstage, emit, EV_RUN_FWD);
        }
        for (int j : ids_upto(i)) {
            bool keep = sch.fwd_save[j];
            for (int t : g.nodes[j].consumers) keep = keep || t > i;
            if (!keep) drop(fstage, j);
        }
        if (sch.fwd_save[i]) {
            if (!held.count(i)) throw PlanError(MONET_INFEASIBLE, "forward pass saves node " + std::to_string(i) + ", which is not in memory");
            ev(EV_SAVE, fstage, i, -1, 0, held[i].second);
        }
    }

    // ---- backward pass
    std::vector<int> last_bop(N + 1, 0);
    for (int k = B; k >= 1; --k) last_bop[g.bops[k].node] = k;   // lowest k of each node wins
    for (int k = B; k >= 1; --k) {
        const Bop &b = g.bops[k];
        const auto &rk = sch.r[k];
        const auto &sk = sch.s[k];
        const int l = sch.stage_impl[k];
        const BwdImpl &im = b.impls[l];
        std::vector<int> D = node_deps(g, k, l);
        auto inD = [&](int j) { return std::find(D.begin(), D.end(), j) != D.end(); };
        for (int i = 1; i <= N; ++i) {
            const Node &n = g.nodes[i];
            auto it = rk.find(i);
            if (it != rk.end() && !n.aux) {
                std::vector<int> emit;
                for (int c : n.aux_children) if (rk.count(c)) emit.push_back(c);
                run_forward(i, it->second, k, emit, EV_RUN_RECOMPUTE);
            }
            for (int j : ids_upto(i)) {
                bool keep = sk.count(j) || inD(j);
                for (int t : g.nodes[j].consumers) keep = keep || (t > i && rk.count(t));
                if (!keep) drop(k, j);
            }
            if (sk.count(i)) {
                if (!held.count(i)) throw PlanError(MONET_INFEASIBLE, "stage " + std::to_string(k) + " saves node " + std::to_string(i) + ", which is not in memory");
                ev(EV_SAVE, k, i, -1, 0, held[i].second);
            }
        }
        const Node &n = g.nodes[b.node];
        std::string who = "backward operator " + std::to_string(k);
        Launch L;
        L.kind = EV_RUN_BWD; L.id = k; L.impl = l;
        begin_launch(chainable(L));
        if (!n.persist) {
            auto gi = grads.find(b.node);
            if (gi == grads.end()) throw PlanError(MONET_BAD_GRAPH, who + " has no incoming gradient");
            L.a[0].region = R_ARENA; L.a[0].off = gi->second.first;
        }
        for (int d : D) fwd_ref(d, who);
        if (!D.empty()) L.a[1] = fwd_ref(D[0], who);
        else if (b.kind.size() > 6 && b.kind.compare(b.kind.size() - 6, 6, "_wgrad") == 0) L.a[1] = fwd_ref(n.ins[0], who);
        uint32_t acc = 0;
        for (int p : grad_positions(g, b)) {
            int j = n.ins[p];
            auto gj = grads.find(j);
            if (gj != grads.end()) acc |= 1u << p;
            else {
                int64_t off = arena_alloc(k, j, T_GRAD, g.nodes[j].bytes);
                grads[j] = {off, g.nodes[j].bytes};
                gj = grads.find(j);
            }
            if (p < 2) { L.a[2 + p].region = R_ARENA; L.a[2 + p].off = gj->second.first; }
        }
        L.flags = acc;
        int64_t wsb = im.ws > 0 ? align_up(im.ws) : 0, wso = 0;
        if (wsb) { wso = arena_alloc(k, k, T_BWS, wsb); L.a[4].region = R_ARENA; L.a[4].off = wso; }
        ev(EV_RUN_BWD, k, k, l, (int)acc, 0);
        L.event = events.size() - 1;
        snapshot();
        launches.push_back(L);
        if (wsb) arena_free(k, k, T_BWS, wso, wsb);
        if (!n.persist && last_bop[b.node] == k) {
            auto gi = grads[b.node];
            grads.erase(b.node);
            arena_free(k, b.node, T_GRAD, gi.first, gi.second);
        }
        for (int j : ids_upto(N))
            if (!sk.count(j)) drop(k, j);
    }
    if (!held.empty() || !grads.empty() || live != 0)
        throw PlanError(MONET_INFEASIBLE, "tensors are left in memory after the last stage");
    exact_peak = peak;
    flush_pending(true);
    dynamic_bytes = arena.high;
}

// ------------------------------------------------------------------ predicted peak from the formulas (Eq. 1, Eq. 5, Eq. 6, C.2)
void Plan::closed_form() {
    const int N = g.N(), B = g.B();
    auto ws_of = [](int64_t ws) { return ws > 0 ? align_up(ws) : (int64_t)0; };
    std::set<int> fsave;
    for (int i = 1; i <= N; ++i) if (sch.fwd_save[i]) fsave.insert(i);
    auto bytes_of_set = [&](const std::set<int> &s) { int64_t t = 0; for (int j : s) t += g.nodes[j].bytes; return t; };
    auto own_out = [&](const Node &n, const FwdImpl &im, const std::vector<int> &emit) {
        int64_t t = (im.inplace || n.persist) ? 0 : n.bytes;
        for (int c : emit) t += g.nodes[c].bytes;
        return t;
    };
    // L-bar_i: earlier tensors read by operator i or a later one
    auto Lbar = [&](int i) {
        std::set<int> s;
        for (int j = 1; j < i; ++j)
            for (int t : g.nodes[j].consumers) if (t >= i) { s.insert(j); break; }
        return s;
    };
    // L-dot_i^k (Appendix B): of those, only what an operator up to the stage's own node reads
    auto Ldot = [&](int i, int last) {
        std::set<int> s;
        for (int j = 1; j < i; ++j)
            for (int t : g.nodes[j].consumers) if (t >= i && t <= last) { s.insert(j); break; }
        return s;
    };
    int64_t best = 0, tight = 0;
    for (int i = 1; i <= N; ++i) {
        const Node &n = g.nodes[i];
        if (n.aux) continue;
        const FwdImpl &im = n.fimpls[sch.fwd_impl[i]];
        std::vector<int> emit;
        for (int c : n.aux_children) if (sch.fwd_save[c]) emit.push_back(c);
        std::set<int> u = Lbar(i);
        for (int j : fsave) if (j < i) u.insert(j);
        best = std::max(best, ws_of(im.ws) + own_out(n, im, emit) + bytes_of_set(u));
    }
    tight = best;
    // gradient tensors: born at the highest stage writing them, gone after the lowest stage of their node
    std::map<int, int> born, dies;
    for (int k = 1; k <= B; ++k) {
        const Bop &b = g.bops[k];
        const Node &n = g.nodes[b.node];
        for (int p : grad_positions(g, b)) born[n.ins[p]] = std::max(born[n.ins[p]], k);
        if (!n.persist && !dies.count(b.node)) dies[b.node] = k;
    }
    for (int k = B; k >= 1; --k) {
        const Bop &b = g.bops[k];
        const BwdImpl &im = b.impls[sch.stage_impl[k]];
        int64_t lhat = 0, yk = 0;
        for (auto &kv : born) {
            if (kv.second > k && k >= dies[kv.first]) lhat += g.nodes[kv.first].bytes;
            if (kv.second == k) yk += g.nodes[kv.first].bytes;
        }
        std::set<int> D;
        for (int d : node_deps(g, k, sch.stage_impl[k])) D.insert(d);
        std::set<int> u = D;
        u.insert(sch.s[k].begin(), sch.s[k].end());
        best = std::max(best, ws_of(im.ws) + yk + lhat + bytes_of_set(u));
        tight = std::max(tight, ws_of(im.ws) + yk + lhat + bytes_of_set(u));
        const auto &enter = sch.entering(k, B, fsave);
        const auto &rk = sch.r[k];
        for (int i = 1; i <= N; ++i) {
            const Node &n = g.nodes[i];
            int64_t later = 0;
            for (int j : enter) if (j > i) later += g.nodes[j].bytes;
            auto it = rk.find(i);
            std::set<int> u2;
            if (it != rk.end() && !n.aux) {
                const FwdImpl &fi = n.fimpls[it->second];
                std::vector<int> emit;
                for (int c : n.aux_children) if (rk.count(c)) emit.push_back(c);
                u2 = Lbar(i);
                for (int j : sch.s[k]) if (j < i) u2.insert(j);
                for (int j : D) if (j < i) u2.insert(j);
                best = std::max(best, ws_of(fi.ws) + own_out(n, fi, emit) + lhat + bytes_of_set(u2) + later);
                std::set<int> u3 = Ldot(i, b.node);
                for (int j : sch.s[k]) if (j < i) u3.insert(j);
                for (int j : D) if (j < i) u3.insert(j);
                tight = std::max(tight, ws_of(fi.ws) + own_out(n, fi, emit) + lhat + bytes_of_set(u3) + later);
            } else {
                for (int j : sch.s[k]) if (j <= i) u2.insert(j);
                for (int j : D) if (j <= i) u2.insert(j);
                best = std::max(best, lhat + bytes_of_set(u2) + later);
                tight = std::max(tight, lhat + bytes_of_set(u2) + later);
            }
        }
    }
    predicted_peak = best;
    predicted_peak_tight = tight;
}

void Plan::build(const std::string &graph_text, const std::string &schedule_text) {
    g.parse(graph_text);
    check_declared_deps(g);
    sch.parse(schedule_text, g);
    validate();
    // constant region: loss scalar, BatchNorm statistics, reduction scratch
    int64_t off = 0;
    loss_off = off; off += kAlign;
    for (int i = 1; i <= g.N(); ++i)
        if (g.nodes[i].op == "bn") {
            bn_stats_off[i] = off;
            off += align_up(2 * g.nodes[i].shape.back() * 4);
        }
    scratch_off = off;
    // holds the partial results of the two-level reductions; the largest user is BatchNorm's forward statistics
    // in groups of 64 rows (2 floats per group and channel: 72 MB for VGG-16's first layers at batch 176)
    scratch_bytes = 96ll << 20;
    off += scratch_bytes;
    persistent_bytes = off;
    lower();
    closed_form();
}

}  // namespace monet
