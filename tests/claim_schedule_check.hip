// Host-only check of the streaming passes' work distribution (csrc/launch.h, csrc/device_common.h): for many
// buffer sizes, grids, chunk sizes and alignment phases, the ranges of claims 0 .. num_chunks-1 must tile
// [0, N) exactly, in address order, every chunk start after the first on a 128-byte line of the reference
// stream and a whole number of iterations from the origin.  Compiled and run by tests/test_claim_schedule.py.
#include <stdio.h>
#include <stdlib.h>
#include "launch.h"
using namespace diloco;
int main() {
    unsigned long long cases = 0, claims_total = 0;
    uint64_t Ns[] = {0, 1, 5, 127, 128, 129, 4095, 4096, 4097, 8191, 100000, 1u << 20, 3000001, 218112000ull, 1276422656ull, 10211381248ull, 729384375ull, (1ull << 32) + 5};
    int cus[] = {1, 4, 256};
    int bpcs[] = {1, 2, 4, 7};
    uint64_t maxit[] = {1, 2, 4, 8, 16, 128};
    for (uint64_t N : Ns) for (int cu : cus) for (int bpc : bpcs) for (uint64_t mi : maxit) for (uint32_t phase : {0u, 1u, 77u, 127u}) {
        Grid g = plan_grid(N, cu, bpc, (unsigned long long*)1, phase, mi);
        const Work& w = g.work;
        uint64_t pos = 0;
        if (w.num_chunks > 40000000ull) continue;       // skip the slowest combos
        for (unsigned long long c = 0; c < w.num_chunks; ++c) {
            Share sh = claim_range(w, c, N);
            if (sh.begin != pos && !(sh.begin >= N && pos >= N)) { printf("gap N=%llu cu=%d bpc=%d mi=%llu phase=%u c=%llu begin=%llu pos=%llu\n", (unsigned long long)N, cu, bpc, (unsigned long long)mi, phase, c, (unsigned long long)sh.begin, (unsigned long long)pos); return 1; }
            if (sh.end < sh.begin && sh.begin < N) { printf("neg\n"); return 1; }
            if (sh.begin < N) {
                if (c > 0 && ((sh.begin + phase) % kAlignElems) != 0) { printf("misaligned chunk start\n"); return 1; }
                if (((sh.begin ? sh.begin - w.origin : 0) % kIter) != 0 && c > 0) { printf("not a multiple of kIter\n"); return 1; }
                pos = sh.end;
            }
        }
        if (pos != N) { printf("coverage N=%llu cu=%d bpc=%d mi=%llu phase=%u: ends at %llu, %llu chunks\n", (unsigned long long)N, cu, bpc, (unsigned long long)mi, phase, (unsigned long long)pos, (unsigned long long)w.num_chunks); return 1; }
        ++cases; claims_total += w.num_chunks;
    }
    // static plan too
    for (uint64_t N : Ns) for (int cu : cus) for (int bpc : bpcs) for (uint32_t phase : {0u, 3u}) {
        Grid g = plan_static(N, cu, bpc, phase);
        uint64_t pos = 0;
        for (unsigned long long c = 0; c < g.work.num_chunks; ++c) { Share sh = claim_range(g.work, c, N); if (sh.begin < N) { if (sh.begin != pos) { printf("static gap\n"); return 1; } pos = sh.end; } }
        if (pos != N) { printf("static coverage N=%llu\n", (unsigned long long)N); return 1; }
        ++cases;
    }
    printf("ok: %llu cases, %llu claims\n", cases, claims_total);
    return 0;
}
