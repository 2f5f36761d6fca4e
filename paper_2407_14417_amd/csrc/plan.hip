// Partitioner / planner of the paper's §3 (host-only): how many experts are 4-bit (Eq. 1 under a throughput
// preference, the task's number under a quality preference), which ones (seeded random choice), and which
// experts stay in device memory (4-bit first).  Documented in include/moemix.h.
#include <vector>

#include "../../include/moemix.h"

namespace {

uint64_t mix64(uint64_t z) {   // splitmix64 finalizer, the generator behind every seeded choice of this library
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

}  // namespace

extern "C" int moe_plan(const moe_plan_request* req, moe_plan_result* res, uint8_t* quantized, uint8_t* resident) {
    if (!req || !res || !quantized || !resident) return MOE_EINVAL;
    const int n = req->num_experts;
    if (n < 1 || req->size_e4 == 0) return MOE_EINVAL;
    if (req->preference != MOE_PREFER_THROUGHPUT && req->preference != MOE_PREFER_QUALITY) return MOE_EINVAL;
    int n4;
    if (req->preference == MOE_PREFER_THROUGHPUT) {
        // Eq. 1: every expert fits in 4-bit form; each promotion to 16-bit costs three more 4-bit sizes
        const uint64_t all4 = req->size_non_expert + (uint64_t)n * req->size_e4;
        uint64_t n16 = 0;
        if (req->mem_gpu > all4) n16 = (req->mem_gpu - all4) / (3 * req->size_e4);
        if (n16 > (uint64_t)n) n16 = (uint64_t)n;
        n4 = n - (int)n16;
    } else {
        n4 = req->num_e4;
        if (n4 < 0 || n4 > n) return MOE_EINVAL;
    }
    // quantized attribute: Fisher-Yates shuffle of the expert indices, the first n4 of the shuffled order are 4-bit
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    const uint64_t key = mix64(mix64(req->seed) + 0x5EED0A5Cull);
    for (int i = n - 1; i > 0; --i) {
        const int j = (int)(mix64(key + (uint64_t)i) % (uint64_t)(i + 1));
        const int t = order[i]; order[i] = order[j]; order[j] = t;
    }
    for (int i = 0; i < n; ++i) quantized[i] = 0;
    for (int i = 0; i < n4; ++i) quantized[order[i]] = 1;
    // location attribute: 4-bit experts first, then 16-bit ones, while the budget lasts
    const uint64_t fixed = req->size_non_expert + req->swap_bytes;
    uint64_t budget = req->mem_gpu > fixed ? req->mem_gpu - fixed : 0;
    res->num_e4 = n4;
    res->num_e16 = n - n4;
    res->resident_e4 = res->resident_e16 = 0;
    res->bytes_resident = req->size_non_expert;
    for (int i = 0; i < n; ++i) resident[i] = 0;
    for (int cls = 1; cls >= 0; --cls) {
        const uint64_t size = cls ? req->size_e4 : req->size_e16;
        for (int i = 0; i < n; ++i) {
            if (quantized[i] != cls) continue;
            if (budget < size) break;
            budget -= size;
            resident[i] = 1;
            res->bytes_resident += size;
            (cls ? res->resident_e4 : res->resident_e16) += 1;
        }
    }
    return MOE_OK;
}
