// Host-side probe of jot_plan_split (the rule that cuts rows into pieces): prints one line per
// case read from stdin, "n_active V target_items align" -> "S chunk".  Built and run by
// tests/test_host_logic.py; makes no HIP call, so it runs without a GPU.
#include <stdio.h>
#include "../paper_2602_11133_amd/csrc/jot_device.h"

int main()
{
    long long n;
    int V, target, align;
    while (scanf("%lld %d %d %d", &n, &V, &target, &align) == 4) {
        const JotSplit sp = jot_plan_split(n, V, target, align);
        printf("%d %d\n", sp.S, sp.chunk);
    }
    return 0;
}
