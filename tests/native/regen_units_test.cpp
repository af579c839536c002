// Host-only unit test of the walk that deals the regeneration units of a step launch out to its
// blocks (csrc/regen_units.hpp): for many list lengths and grid shapes every unit must be taken
// exactly once, and only by blocks that exist.  Built with g++ and run by tests/test_native_checks.py.
#include <cstdio>
#include <vector>

#include "../../paper_2402_16801_amd/csrc/regen_units.hpp"

static int failures = 0;
static void expect(bool cond, const char* what, unsigned a, unsigned b, unsigned c)
{
    if (!cond && failures < 10) std::printf("FAILED: %s (count %u, regeneration blocks per sub-list %u, step blocks %u)\n", what, a, b, c);
    if (!cond) ++failures;
}

int main()
{
    using namespace cx;
    unsigned long cases = 0;
    const unsigned per_subs[] = { 2, 4, 16, 32, 64 };
    const unsigned nqs[] = { 0, 1, 2, 3, 16, 63, 64, 65, 256 };
    for (unsigned per_sub : per_subs)
        for (unsigned nq : nqs)
            for (unsigned count = 0; count <= 700; count += (count < 70 ? 1 : 37)) {
                if (nq == 0 && count != 0) continue;      // nobody appends to a sub-list without step blocks
                const unsigned units = 2 * count;
                std::vector<int> taken(units, 0);
                unsigned longest = 0;
                for (int helper = 0; helper < 2; ++helper)
                    for (unsigned index = 0; index < (helper ? nq : per_sub); ++index) {
                        unsigned steps = 0, last = 0;
                        for (UnitWalk w = first_unit(helper, index, per_sub); w.u < units; w = next_unit(w, helper, index, per_sub, nq)) {
                            expect(steps == 0 || w.u > last, "a block's units come in rising order", count, per_sub, nq);
                            last = w.u;
                            ++taken[w.u];
                            if (++steps > units) { expect(false, "the walk ends", count, per_sub, nq); break; }
                        }
                        if (helper) expect((steps > 0) == (first_helper_unit(index, per_sub) < units), "first_helper_unit says whether a step block has work", count, per_sub, nq);
                        if (steps > longest) longest = steps;
                    }
                bool once = true;
                for (unsigned u = 0; u < units; ++u) once = once && taken[u] == 1;
                expect(once, "every unit is taken exactly once", count, per_sub, nq);
                // nobody gets more than the head rounds plus an even share of the tail
                const unsigned head = HEAD_ROUNDS * per_sub, tail = units > head ? units - head : 0, workers = nq + per_sub;
                expect(longest <= HEAD_ROUNDS + (tail + workers - 1) / workers, "the tail is shared evenly", count, per_sub, nq);
                ++cases;
            }
    // the headline shape: 1,024 step blocks, 256 regeneration blocks, about 23 finished episodes per sub-list
    {
        const unsigned per_sub = 16, nq = 64, count = 23;
        unsigned helpers_with_work = 0;
        for (unsigned q = 0; q < nq; ++q) helpers_with_work += first_helper_unit(q, per_sub) < 2 * count;
        expect(helpers_with_work == 2 * count - HEAD_ROUNDS * per_sub, "the step blocks with the lowest numbers take the tail, one unit each", count, per_sub, nq);
    }
    if (failures) std::printf("regen_units_test: %d failures\n", failures);
    else std::printf("regen_units_test: ok (%lu shapes)\n", cases);
    return failures ? 1 : 0;
}
