// Host-side check of the operand layouts that kernels and host code share (no GPU call).
// Built and run by tests/test_host_abi.py.
#include <cstdio>
#include <set>
#include <vector>

#include "../paper_2601_11822_amd/csrc/common.h"

static int fails = 0;
#define CHECK(c, ...) do { if (!(c)) { if (fails++ < 10) { std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } } } while (0)

int main() {
    // fragment-packed operand: block (kb, t) is 512 elements, lane h*32 + r of it holds row 32t + r, k 16kb + 8h .. +8
    const int Ms[] = {1, 31, 32, 64, 65, 100, 2048}, Ks[] = {16, 48, 256, 1376};
    for (int M : Ms)
        for (int K : Ks) {
            const int Mt = packed_mt(M), Kb = (K + 15) / 16;
            CHECK(Mt >= 2 && Mt * 32 >= M, "packed_mt(%d) = %d", M, Mt);
            std::set<size_t> seen;
            for (int m = 0; m < Mt * 32; ++m)
                for (int k = 0; k < Kb * 16; k += 8) {
                    const size_t off = packed_offset(m, k, Mt);
                    CHECK(off % 8 == 0 && off / 8 < (size_t)Kb * Mt * 64, "offset out of range m=%d k=%d", m, k);
                    CHECK(seen.insert(off).second, "offset reused m=%d k=%d", m, k);
                    const size_t blk = off / 512, lane = (off % 512) / 8;
                    CHECK(blk == (size_t)(k / 16) * Mt + m / 32, "block of m=%d k=%d", m, k);
                    CHECK(lane == (size_t)((k / 8) % 2) * 32 + m % 32, "lane of m=%d k=%d", m, k);
                }
            CHECK(seen.size() == (size_t)Kb * Mt * 64, "not a bijection M=%d K=%d", M, K);
        }
    // K pool: within one (block, kv head) the 16 token slots x hd dims map one-to-one onto 16*hd elements,
    // 8 dims of one slot stay together, and slots 4-7 and 8-11 trade places
    for (int hd : {64, 128}) {
        std::set<int> seen;
        for (int t = 0; t < 16; ++t)
            for (int d = 0; d < hd; d += 8) {
                const int off = kpool_chunk_offset(t, d);
                CHECK(off % 8 == 0 && off >= 0 && off < 16 * hd, "kpool offset out of range t=%d d=%d", t, d);
                CHECK(seen.insert(off).second, "kpool offset reused t=%d d=%d", t, d);
                const int prow = (off / 8) % 16, grp = off / 128;
                const int want = (t < 4 || t >= 12) ? t : (t < 8 ? t + 4 : t - 4);
                CHECK(prow == want, "permuted row of slot %d is %d", t, prow);
                CHECK(grp == (d / 32) * 4 + (d / 8) % 4, "dim group of d=%d", d);
            }
        CHECK((int)seen.size() == 2 * hd, "kpool not a bijection hd=%d", hd);
    }
    if (fails) { std::printf("%d checks failed\n", fails); return 1; }
    std::printf("layouts ok\n");
    return 0;
}
