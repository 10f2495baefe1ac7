// Test infrastructure: drives the host side of the library (shape checking, the cost model, the
// tuners of Algorithm 1 and the exact search, plan queries, argument checking) through the C ABI in
// a build instrumented with AddressSanitizer and UndefinedBehaviorSanitizer.  No GPU is touched:
// the networks are shape-only and the kernel launchers are replaced by the stand-ins below, which
// fail if they are ever reached.
//
// Input (stdin), whitespace separated:
//   net <in_h> <in_w> <in_c> <n>   followed by n layers of 11 integers
//                                  (op cin cout kh kw stride pad has_bias act input_from residual_from)
//   plan <batch> <mode> <fixed_budget> <max_lds_bytes>
//   manual <batch> <k> <last_0> <budget_0> ... <last_k-1> <budget_k-1>
//   costs <batch>                  dlf_group_cost over every (first, last, budget)
//   badargs                        calls that must be rejected
// Output: one line per command; exit status 0 unless a call misbehaves.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <iostream>
#include <string>
#include <vector>

#include "../include/dlf.h"
#include "../paper_2011_05630_amd/csrc/dlf_internal.h"

extern "C" {
static int unreachable_launch(const char* what)
{
    std::fprintf(stderr, "launcher %s reached in a build without device code\n", what);
    std::abort();
}
int dlf_launch_group(const DlfGroupArgs*, int, int, int, void*) { return unreachable_launch("group"); }
int dlf_launch_fc(const DlfFcArgs*, void*) { return unreachable_launch("fc"); }
int dlf_launch_gap(const DlfGapArgs*, void*) { return unreachable_launch("gap"); }
int dlf_launch_pw(const DlfPwArgs*, int, int, void*) { return unreachable_launch("pw"); }
int dlf_launch_c3(const DlfC3Args*, int, int, int, void*) { return unreachable_launch("c3"); }
int dlf_launch_c3_i8(const DlfC3Args*, int, int, int, void*) { return unreachable_launch("c3_i8"); }
int dlf_launch_pw_i8(const DlfPwArgs*, int, int, void*) { return unreachable_launch("pw_i8"); }
int dlf_launch_dw(const DlfDwArgs*, int, void*) { return unreachable_launch("dw"); }
int dlf_launch_dwpw(const DlfDwPwArgs*, int, int, void*) { return unreachable_launch("dwpw"); }
int dlf_launch_dwt(const DlfDwtArgs*, int, int, void*) { return unreachable_launch("dwt"); }
int dlf_launch_dws(const DlfDwsArgs*, int, int, void*) { return unreachable_launch("dws"); }
int dlf_launch_c3s(const DlfC3sArgs*, int, int, void*) { return unreachable_launch("c3s"); }
int dlf_launch_c3pw(const DlfC3PwArgs*, int, int, void*) { return unreachable_launch("c3pw"); }
int dlf_launch_bneck(const DlfBnArgs*, int, int, void*) { return unreachable_launch("bneck"); }
int dlf_kernels_init(void) { return unreachable_launch("init"); }
void dlf_next_launch_events(void*, void*) { (void)unreachable_launch("events"); }
}

static const int32_t kBudgets[4] = {32, 64, 128, 256};

static void die(const char* what)
{
    std::fprintf(stderr, "driver: %s (%s)\n", what, dlf_last_error());
    std::exit(3);
}

static void show_plan(const char* tag, dlf_plan_t* plan)
{
    const int32_t ng = dlf_plan_num_groups(plan);
    uint64_t total = 0;
    std::printf("%s %d groups:", tag, ng);
    for (int32_t g = 0; g < ng; ++g) {
        int32_t first, last, budget, th, tw;
        uint64_t cost;
        if (dlf_plan_group(plan, g, &first, &last, &budget, &th, &tw, &cost) != DLF_OK) die("dlf_plan_group");
        if (dlf_plan_group(plan, g, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) != DLF_OK)
            die("dlf_plan_group with null outputs");
        total += cost;
        std::printf(" [%d,%d]@%d", first, last, budget);
    }
    if (dlf_plan_group(plan, ng, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == DLF_OK)
        die("dlf_plan_group accepted an index past the end");
    std::printf(" cost %llu ws %zu\n", (unsigned long long)total, dlf_plan_workspace_bytes(plan));
}

int main()
{
    std::vector<dlf_layer_desc> layers;
    dlf_net_t* net = nullptr;
    std::string cmd;
    while (std::cin >> cmd) {
        if (cmd == "net") {
            int32_t h, w, c, n;
            std::cin >> h >> w >> c >> n;
            layers.assign((size_t)n, dlf_layer_desc{});
            for (auto& L : layers) {
                std::cin >> L.op >> L.cin >> L.cout >> L.kh >> L.kw >> L.stride >> L.pad >> L.has_bias >> L.act >>
                    L.input_from >> L.residual_from;
                L.weight = nullptr;
                L.bias = nullptr;
            }
            if (!std::cin) die("malformed net");
            if (net) dlf_net_destroy(net);
            net = nullptr;
            const dlf_status s = dlf_net_create(layers.data(), n, h, w, c, &net);
            std::printf("net %d layers: %s\n", n, dlf_status_string(s));
            if (s == DLF_OK) {
                if (dlf_net_num_layers(net) != n) die("dlf_net_num_layers");
                for (int32_t i = 0; i < n; ++i) {
                    int32_t oh, ow, oc;
                    uint64_t ops;
                    if (dlf_net_layer_info(net, i, &oh, &ow, &oc, &ops) != DLF_OK) die("dlf_net_layer_info");
                }
                int32_t oh;
                if (dlf_net_layer_info(net, n, &oh, nullptr, nullptr, nullptr) == DLF_OK)
                    die("dlf_net_layer_info accepted an index past the end");
            } else {
                net = nullptr;
            }
        } else if (cmd == "plan") {
            int32_t batch, mode, fixed, lds;
            std::cin >> batch >> mode >> fixed >> lds;
            if (!net) die("plan without a net");
            dlf_tuner_opts o;
            std::memset(&o, 0, sizeof o);
            o.mode = mode;
            o.budgets = kBudgets;
            o.n_budgets = 4;
            o.fixed_budget = fixed;
            o.max_lds_bytes = lds;
            dlf_plan_t* plan = nullptr;
            const dlf_status s = dlf_plan(net, batch, &o, &plan);
            if (s != DLF_OK) {
                std::printf("plan mode %d: %s\n", mode, dlf_status_string(s));
                continue;
            }
            show_plan("plan", plan);
            // a shape-only network must refuse to run, before any launcher is reached (a network of
            // pooling layers alone has no weights to miss and would run)
            bool weighted = false;
            for (const auto& L : layers) weighted = weighted || L.op == DLF_CONV || L.op == DLF_DWCONV || L.op == DLF_FC;
            if (!weighted) { dlf_plan_destroy(plan); continue; }
            if (dlf_run(plan, &o, &o, nullptr) == DLF_OK) die("dlf_run accepted a shape-only network");
            if (dlf_run_noalloc(plan, &o, &o, nullptr) == DLF_OK) die("dlf_run_noalloc accepted a shape-only network");
            dlf_plan_destroy(plan);
        } else if (cmd == "manual") {
            int32_t batch, k;
            std::cin >> batch >> k;
            std::vector<int32_t> last((size_t)k), bud((size_t)k);
            for (int32_t i = 0; i < k; ++i) std::cin >> last[(size_t)i] >> bud[(size_t)i];
            if (!net) die("manual without a net");
            dlf_tuner_opts o;
            std::memset(&o, 0, sizeof o);
            o.mode = DLF_TUNER_MANUAL;
            o.manual_group_last = last.data();
            o.manual_budget = bud.data();
            o.manual_n = k;
            dlf_plan_t* plan = nullptr;
            const dlf_status s = dlf_plan(net, batch, &o, &plan);
            if (s != DLF_OK) {
                std::printf("manual: %s\n", dlf_status_string(s));
                continue;
            }
            show_plan("manual", plan);
            dlf_plan_destroy(plan);
        } else if (cmd == "costs") {
            int32_t batch;
            std::cin >> batch;
            if (!net) die("costs without a net");
            const int32_t n = dlf_net_num_layers(net);
            long feasible = 0, infeasible = 0;
            for (int32_t f = 0; f < n; ++f)
                for (int32_t l = f; l < n && l < f + 8; ++l)
                    for (int32_t b : kBudgets) {
                        uint64_t c = 0;
                        const dlf_status s = dlf_group_cost(net, batch, f, l, b, 0, &c);
                        if (s == DLF_OK) ++feasible;
                        else if (s == DLF_ERR_INFEASIBLE) ++infeasible;
                        else die("dlf_group_cost");
                    }
            std::printf("costs %ld feasible %ld infeasible\n", feasible, infeasible);
        } else if (cmd == "badargs") {
            if (!net) die("badargs without a net");
            dlf_plan_t* plan = nullptr;
            dlf_net_t* other = nullptr;
            uint64_t c;
            int bad = 0;
            bad += dlf_net_create(nullptr, 3, 8, 8, 8, &other) == DLF_OK;
            bad += dlf_net_create(layers.data(), 0, 8, 8, 8, &other) == DLF_OK;
            bad += dlf_net_create(layers.data(), (int32_t)layers.size(), -1, 8, 8, &other) == DLF_OK;
            bad += dlf_net_create(layers.data(), (int32_t)layers.size(), 8, 8, 8, nullptr) == DLF_OK;
            bad += dlf_plan(nullptr, 1, nullptr, &plan) == DLF_OK;
            bad += dlf_plan(net, 0, nullptr, &plan) == DLF_OK;
            bad += dlf_plan(net, 1, nullptr, nullptr) == DLF_OK;
            bad += dlf_group_cost(net, 1, -1, 0, 64, 0, &c) == DLF_OK;
            bad += dlf_group_cost(net, 1, 1, 0, 64, 0, &c) == DLF_OK;
            bad += dlf_group_cost(net, 1, 0, dlf_net_num_layers(net), 64, 0, &c) == DLF_OK;
            bad += dlf_group_cost(net, 1, 0, 0, 0, 0, &c) == DLF_OK;
            bad += dlf_group_cost(net, 1, 0, 0, 64, 0, nullptr) == DLF_OK;
            dlf_tuner_opts o;
            std::memset(&o, 0, sizeof o);
            o.mode = 99;
            bad += dlf_plan(net, 1, &o, &plan) == DLF_OK;
            o.mode = DLF_TUNER_MANUAL;          // manual mode without lists
            bad += dlf_plan(net, 1, &o, &plan) == DLF_OK;
            const int32_t neg[2] = {-3, 7};
            o.mode = DLF_TUNER_DP;
            o.budgets = neg;
            o.n_budgets = 2;
            bad += dlf_plan(net, 1, &o, &plan) == DLF_OK;
            // the quantised layer: shape-only layers of both filter sizes over a range of maps, and rejected sizes
            for (int32_t k = 1; k <= 3; k += 2)
                for (int32_t hw : {1, 7, 14, 28, 56, 112})
                    for (int32_t ch : {64, 128, 512}) {
                        dlf_i8conv_t* q = nullptr;
                        if (dlf_i8conv_create(3, hw, hw + 1, ch, ch + 16, k, 1, (k == 3 && hw > 1) ? 1 : 0, nullptr, nullptr, nullptr, 0, &q) != DLF_OK)
                            die("dlf_i8conv_create");
                        int32_t th, tw, sh, gr;
                        uint64_t ops;
                        if (dlf_i8conv_info(q, &th, &tw, &sh, &gr, &ops) != DLF_OK || gr < 8 || (gr & 7) || th < 1 || tw < 1)
                            die("dlf_i8conv_info");
                        bad += dlf_i8conv_run(q, layers.data(), layers.data(), nullptr) == DLF_OK;     // no weights
                        dlf_i8conv_destroy(q);
                    }
            {
                dlf_i8conv_t* q = nullptr;
                bad += dlf_i8conv_create(1, 8, 8, 64, 64, 3, 0, 0, nullptr, nullptr, nullptr, 0, nullptr) == DLF_OK;
                bad += dlf_i8conv_create(1, 8, 8, 32, 64, 3, 0, 0, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;
                bad += dlf_i8conv_create(1, 8, 8, 64, 8, 1, 0, 0, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;
                bad += dlf_i8conv_create(1, 8, 8, 64, 64, 2, 0, 0, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;
                bad += dlf_i8conv_create(1, -8, 8, 64, 64, 3, 0, 0, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;
                bad += dlf_i8conv_create(1 << 20, 1 << 10, 1 << 10, 64, 64, 3, 0, 0, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;
                bad += dlf_i8conv_create(1, 8, 8, 64, 64, 1, 0, 1, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;     // pool behind a 1x1
                bad += dlf_i8conv_create(1, 8, 8, 64, 64, 3, 0, 2, nullptr, nullptr, nullptr, 0, &q) == DLF_OK;
                bad += dlf_i8conv_info(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == DLF_OK;
                dlf_i8conv_destroy(nullptr);
            }
            dlf_net_destroy(nullptr);
            dlf_plan_destroy(nullptr);
            if (bad) die("a bad argument was accepted");
            std::printf("badargs rejected\n");
        } else {
            die("unknown command");
        }
    }
    if (net) dlf_net_destroy(net);
    return 0;
}
