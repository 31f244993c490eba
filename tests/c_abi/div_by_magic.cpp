// The reciprocal division the kernels use to split a lane's combination into digits
// (jsv::div_by_magic, jsv::magic_of) against / and %: every divisor a task's list can have,
// the boundary dividends of each, and random ones.  Built with g++ (the header is plain C++)
// and run by tests/test_host_abi.py.
#include <cstdint>
#include <cstdio>

#include "../../paper_2603_08797_amd/csrc/jsv_device.h"

int main()
{
    uint64_t state = 0x9E3779B97F4A7C15ull, checked = 0, bad = 0;
    auto next = [&]() { state += 0x9E3779B97F4A7C15ull; uint64_t z = state; z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
                        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; return z ^ (z >> 31); };
    auto check = [&](uint32_t x, uint32_t k) {
        uint32_t r = 0;
        const uint32_t q = jsv::div_by_magic(x, k, jsv::magic_of(k), &r);
        ++checked;
        if (q != x / k || r != x % k) { if (bad++ < 5) std::printf("x=%u k=%u: got %u rem %u\n", x, k, q, r); }
    };
    for (uint32_t k = 1; k <= 2 * (uint32_t)jsv::MAXC; ++k) {
        const uint32_t top = 0xFFFFFFFFu / k * k;          // the largest multiple of k
        const uint32_t edge[] = {0u, 1u, k - 1, k, k + 1, 2 * k - 1, 2 * k, top - 1, top, top + (k > 1 ? 1u : 0u),
                                 0x7FFFFFFFu, 0x80000000u, 0xFFFFFFFEu, 0xFFFFFFFFu};
        for (uint32_t x : edge) check(x, k);
        for (int i = 0; i < 500; ++i) check((uint32_t)next(), k);
        for (int i = 0; i < 100; ++i) check((uint32_t)(next() % ((uint64_t)k * k + 1)), k);
    }
    for (int i = 0; i < 2000000; ++i) check((uint32_t)next(), (uint32_t)(next() % 0xFFFFFFFFull) + 1u);   // any divisor at all
    std::printf(bad ? "FAILED (%llu of %llu)\n" : "div by magic ok (%llu checked)\n", (unsigned long long)(bad ? bad : checked), (unsigned long long)checked);
    return bad ? 1 : 0;
}
