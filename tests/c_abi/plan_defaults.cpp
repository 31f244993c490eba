// A freshly declared jsv::Plan must have every mode switch off and every pointer null, so that
// a call site which forgets a field cannot send a kernel into a mode it did not ask for.
// Built with g++ (the header is plain C++, no HIP needed) and run by tests/test_host_abi.py.
#include <cstdio>
#include <cstring>
#include <new>

#include "../../paper_2603_08797_amd/csrc/jsv_device.h"

int main()
{
    // construct over memory full of ones: whatever a constructor does not set stays visible
    alignas(jsv::Plan) unsigned char raw[sizeof(jsv::Plan)];
    std::memset(raw, 0xFF, sizeof raw);
    const jsv::Plan* pl = new (raw) jsv::Plan;
    int bad = 0;
#define EXPECT_ZERO(field) if (pl->field != 0) { std::printf("Plan::" #field " is not 0\n"); ++bad; }
#define EXPECT_NULL(field) if (pl->field != nullptr) { std::printf("Plan::" #field " is not null\n"); ++bad; }
    EXPECT_ZERO(objective) EXPECT_ZERO(mix) EXPECT_ZERO(bounds) EXPECT_ZERO(mix_cells)
    EXPECT_ZERO(n_inst) EXPECT_ZERO(t_max) EXPECT_ZERO(k_max) EXPECT_ZERO(c_max)
    EXPECT_ZERO(grid) EXPECT_ZERO(lanes_wanted) EXPECT_ZERO(cut) EXPECT_ZERO(pair_cap) EXPECT_ZERO(pair_pad)
    EXPECT_NULL(graphs) EXPECT_NULL(inst) EXPECT_NULL(entries) EXPECT_NULL(rep) EXPECT_NULL(cost)
    EXPECT_NULL(k32) EXPECT_NULL(quads) EXPECT_NULL(partial) EXPECT_NULL(partial_obj)
    EXPECT_NULL(results) EXPECT_NULL(summary) EXPECT_NULL(cell_acc) EXPECT_NULL(cell_id)
    EXPECT_NULL(cell_pm) EXPECT_NULL(cell_list) EXPECT_NULL(bound) EXPECT_NULL(tile_begin)
    EXPECT_NULL(pairs) EXPECT_NULL(best_obj)
    // the members listed above are all there is: no padding, nothing forgotten
    const size_t listed = 12 * sizeof(void*) + 12 * sizeof(uint32_t) + 4 * sizeof(void*) + sizeof(uint64_t) + 3 * sizeof(void*);
    if (listed != sizeof(jsv::Plan)) { std::printf("Plan has members this test does not know: %zu vs %zu\n", listed, sizeof(jsv::Plan)); ++bad; }
    std::printf(bad ? "FAILED\n" : "plan defaults ok\n");
    return bad ? 1 : 0;
}
