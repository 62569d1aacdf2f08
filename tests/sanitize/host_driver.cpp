// Drives the host-side entry points of the library from a script on stdin and prints what they return, one line
// per command.  Built with -fsanitize=address,undefined against a build of the library whose host code carries
// the same instrumentation; every array handed to the library is a heap block of exactly its own size.  No
// command touches a GPU: contexts are created with LORA_CREATE_HOST_ONLY.
//
//   ctx  <n_slots> <max_rank> <max_adapter_id> <n_layers> <n_proj> (<d_in> <d_out>)*      -> ctx <status>
//   load <n_in_use> <id>* <n_req> (<id> <rank> <slot>)*        -> load <status> (<slot>:<copied>)*   then   state <id>*
//   ctxp <n_slots> <max_rank> <max_adapter_id> <n_layers> <n_pages> <n_proj> (<d_in> <d_out>)*   -> ctx <status>  (slots over a pool of pages)
//   pages                                                      -> pages <first page>*
//   map  <n_ids>                                               -> map <slot>*
//   slab <n_slots> <max_rank> <max_tokens> <n_layers> <n_proj> (<d_in> <d_out>)*          -> slab <bytes>
//   str  <status>                                              -> str <text>
//   bucket                                                     -> bucket <status>      (device work on a host-only context)
//   prio <n> (<size> <rate>)*                                  -> prio <status> <index>*
//   place <n_gpus> <cap> <n> (<size> <rate>)*                  -> place <status> <gpu>* | <a_max>*
//
// The predictors of `place` (the library takes them from its caller): throughput = min(sum of rates, cap) -
// a_max / 1024, starvation = (sum of rate * size > 8 * cap) or (n > a_max); sums in the order given.
#include "../../include/lora_mi355.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <iostream>
#include <memory>
#include <string>
#include <vector>

namespace {

struct Law {
    double cap;
};

double thr(void* user, int32_t n, const int32_t*, const double* rates, int32_t a_max)
{
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += rates[i];
    return std::min(sum, static_cast<Law*>(user)->cap) - a_max / 1024.0;
}

int32_t starves(void* user, int32_t n, const int32_t* sizes, const double* rates, int32_t a_max)
{
    double load = 0.0;
    for (int32_t i = 0; i < n; ++i) load += rates[i] * sizes[i];
    return (load > 8.0 * static_cast<Law*>(user)->cap || n > a_max) ? 1 : 0;
}

// exactly n elements on the heap (one, untouched, for n = 0)
template <typename T>
std::unique_ptr<T[]> block(size_t n)
{
    return std::unique_ptr<T[]>(new T[n ? n : 1]());
}

template <typename T>
T next(std::istream& in)
{
    T v{};
    if (!(in >> v)) {
        std::fprintf(stderr, "host_driver: truncated script\n");
        std::exit(3);
    }
    return v;
}

struct Shapes {
    int32_t n_proj = 0;
    std::unique_ptr<lora_proj_shape[]> proj;
};

Shapes read_shapes(std::istream& in)
{
    Shapes s;
    s.n_proj = next<int32_t>(in);
    s.proj = block<lora_proj_shape>(std::max(0, s.n_proj));
    for (int32_t p = 0; p < s.n_proj; ++p) {
        s.proj[p].d_in = next<int32_t>(in);
        s.proj[p].d_out = next<int32_t>(in);
    }
    return s;
}

}  // namespace

int main()
{
    lora_ctx* ctx = nullptr;
    int32_t n_slots = 0;
    std::string cmd;
    while (std::cin >> cmd) {
        if (cmd == "ctx" || cmd == "ctxp") {
            if (ctx) lora_destroy(ctx);
            ctx = nullptr;
            lora_config cfg{};
            cfg.n_slots = n_slots = next<int32_t>(std::cin);
            cfg.max_rank = next<int32_t>(std::cin);
            cfg.max_adapter_id = next<int32_t>(std::cin);
            cfg.n_layers = next<int32_t>(std::cin);
            if (cmd == "ctxp") cfg.n_pages = next<int32_t>(std::cin);
            Shapes s = read_shapes(std::cin);
            cfg.n_proj = s.n_proj;
            cfg.proj = s.proj.get();
            cfg.max_tokens = 16;
            cfg.flags = LORA_CREATE_HOST_ONLY;
            const lora_status st = lora_create(&cfg, &ctx);
            std::printf("ctx %d\n", (int)st);
            if (st != LORA_OK) ctx = nullptr;
        } else if (cmd == "load") {
            const int32_t n_in_use = next<int32_t>(std::cin);
            auto in_use = block<int32_t>(n_in_use);
            for (int32_t i = 0; i < n_in_use; ++i) in_use[i] = next<int32_t>(std::cin);
            const int32_t n = next<int32_t>(std::cin);
            auto d = block<lora_adapter_desc>(n);
            for (int32_t i = 0; i < n; ++i) {
                d[i].adapter_id = next<int32_t>(std::cin);
                d[i].rank = next<int32_t>(std::cin);
                d[i].slot = next<int32_t>(std::cin);
                d[i].scale = 1.0f;
            }
            const lora_status st = lora_slots_load(ctx, n, d.get(), in_use.get(), n_in_use, nullptr);
            std::printf("load %d", (int)st);
            if (st == LORA_OK)
                for (int32_t i = 0; i < n; ++i) std::printf(" %d:%d", d[i].slot, d[i].copied);
            std::printf("\nstate");
            for (int32_t s = 0; s < n_slots; ++s) std::printf(" %d", lora_slot_adapter(ctx, s));
            std::printf("\n");
        } else if (cmd == "pages") {
            std::printf("pages");
            for (int32_t s = 0; s < n_slots; ++s) std::printf(" %d", lora_slot_first_page(ctx, s));
            std::printf("\n");
        } else if (cmd == "map") {
            const int32_t n_ids = next<int32_t>(std::cin);
            std::printf("map");
            for (int32_t i = 0; i < n_ids; ++i) std::printf(" %d", lora_slot_of(ctx, i));
            std::printf("\n");
        } else if (cmd == "slab") {
            lora_config cfg{};
            cfg.n_slots = next<int32_t>(std::cin);
            cfg.max_rank = next<int32_t>(std::cin);
            cfg.max_tokens = next<int32_t>(std::cin);
            cfg.n_layers = next<int32_t>(std::cin);
            Shapes s = read_shapes(std::cin);
            cfg.n_proj = s.n_proj;
            cfg.proj = s.proj.get();
            cfg.max_adapter_id = 63;
            std::printf("slab %zu\n", lora_slab_bytes(&cfg));
        } else if (cmd == "str") {
            std::printf("str %s\n", lora_status_string((lora_status)next<int32_t>(std::cin)));
        } else if (cmd == "bucket") {
            lora_segments seg{};
            std::printf("bucket %d\n", (int)lora_bucket(ctx, nullptr, 0, LORA_BUCKET_SORTED, &seg, nullptr));
        } else if (cmd == "prio" || cmd == "place") {
            Law law{0.0};
            int32_t n_gpus = 0;
            if (cmd == "place") {
                n_gpus = next<int32_t>(std::cin);
                law.cap = next<double>(std::cin);
            }
            const int32_t n = next<int32_t>(std::cin);
            auto size = block<int32_t>(n);
            auto rate = block<double>(n);
            for (int32_t i = 0; i < n; ++i) {
                size[i] = next<int32_t>(std::cin);
                rate[i] = next<double>(std::cin);
            }
            if (cmd == "prio") {
                auto order = block<int32_t>(n);
                const lora_status st = lora_priority_sorting(n, size.get(), rate.get(), order.get());
                std::printf("prio %d", (int)st);
                if (st == LORA_OK)
                    for (int32_t i = 0; i < n; ++i) std::printf(" %d", order[i]);
                std::printf("\n");
            } else {
                auto gpu_of = block<int32_t>(n);
                auto a_max = block<int32_t>(std::max(0, n_gpus));
                const lora_status st =
                    lora_place_adapters(n, size.get(), rate.get(), n_gpus, thr, starves, &law, gpu_of.get(), a_max.get());
                std::printf("place %d", (int)st);
                if (st == LORA_OK) {
                    for (int32_t i = 0; i < n; ++i) std::printf(" %d", gpu_of[i]);
                    std::printf(" |");
                    for (int32_t g = 0; g < n_gpus; ++g) std::printf(" %d", a_max[g]);
                }
                std::printf("\n");
            }
        } else {
            std::fprintf(stderr, "host_driver: unknown command %s\n", cmd.c_str());
            return 2;
        }
    }
    if (ctx) lora_destroy(ctx);
    return 0;
}
