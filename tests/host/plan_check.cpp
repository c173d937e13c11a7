// Host-side check of the work-split arithmetic the output-projection kernels and the kernels behind
// them share (plan_rows, splits_of in the library's internal header): compiled for the host only and
// run by tests/test_host_plan.py.  Prints "ok" or the first violated property.
#include <stdio.h>

#include "rnnlm_internal.h"

using namespace rnnlm;

#define REQUIRE(cond, ...)                       \
    do {                                         \
        if (!(cond)) {                           \
            printf("FAILED %s: ", #cond);        \
            printf(__VA_ARGS__);                 \
            printf("\n");                        \
            return 1;                            \
        }                                        \
    } while (0)

int main() {
    const int group_rows_of[] = {128, 256}, wg_of[] = {1, 4, 32, 64}, cap_of[] = {1, 2, 5, 10, 32, 40, 1000};
    for (int group_rows : group_rows_of)
        for (int wg : wg_of)
            for (int cap : cap_of)
                for (int B = 0; B <= 6000; B += (B < 700 ? 1 : 37)) {
                    const RowPlan p = plan_rows(B, group_rows, wg, cap);
                    REQUIRE(p.RG >= 1 && (long long)p.RG * group_rows >= B, "B=%d rows=%d: RG=%d", B, group_rows, p.RG);
                    REQUIRE(B <= group_rows || (p.RG - 1) * group_rows < B, "B=%d rows=%d: RG=%d too many", B, group_rows, p.RG);
                    REQUIRE(p.Sx >= 1 && p.Sx <= cap && p.Sx <= kMaxSplits / kXcds, "B=%d wg=%d cap=%d: Sx=%d", B, wg, cap, p.Sx);
                    REQUIRE(p.S == kXcds * p.Sx && p.S <= kMaxSplits, "S=%d Sx=%d", p.S, p.Sx);
                    // the items of an XCD fit its workgroups in one round whenever they can
                    REQUIRE(p.RG * p.Sx <= wg || p.Sx == 1, "B=%d wg=%d: RG=%d Sx=%d", B, wg, p.RG, p.Sx);
                    // what the kernel behind derives is what the output projection used
                    const SplitInfo si = {0, wg, group_rows, cap, 0};
                    REQUIRE(splits_of(si, B) == p.S, "B=%d: splits_of=%d S=%d", B, splits_of(si, B), p.S);
                    // a kernel that streams the weights for few rows leaves one partial per workgroup
                    if (kXcds * wg <= kMaxSplits) {
                        const SplitInfo ss = {0, wg, group_rows, cap, 64};
                        const int s = splits_of(ss, B);
                        REQUIRE(s == ((B > 0 && B <= 64) ? kXcds * wg : p.S), "B=%d wg=%d: streamed splits %d", B, wg, s);
                        REQUIRE(s <= kMaxSplits, "B=%d: %d partials", B, s);
                    }
                }
    for (int S = 1; S <= kMaxSplits; ++S)
        for (int B = 0; B < 3000; B += 97) REQUIRE(splits_of(fixed_split_info(S), B) == S, "fixed S=%d B=%d", S, B);
    // the staged kernel's plan: 256 rows per group, every group gets the same number of splits
    for (int B = 1; B <= 5000; ++B) {
        const StagedPlan p = staged_plan(B, 32);
        REQUIRE(p.RG == (B + kStagedRows - 1) / kStagedRows && p.S == kXcds * p.Sx, "staged B=%d", B);
    }
    // cutting `units` blocks into `parts` splits: the 32-bit form equals floor(index * units / parts)
    const int units_of[] = {1, 7, 63, 64, 255, 256, 257, 2048, 6250, 31251, 1 << 20, (1 << 25) + 3, 0x7FFFFFFF};
    for (int units : units_of)
        for (int parts = 1; parts <= kMaxSplits; ++parts)
            for (int index = 0; index <= parts; ++index) {
                const long long want = ((long long)index * units) / parts;
                REQUIRE(part_begin(index, units, parts) == (int)want, "part_begin(%d, %d, %d) = %d, want %lld", index, units,
                        parts, part_begin(index, units, parts), want);
            }
    printf("ok\n");
    return 0;
}
