// Host-side check of the LDS tile layouts in csrc/va_device.h (no GPU needed): built and run by
// tests/test_abi_and_host.py.  For every head_dim it verifies, on the index functions the kernels use,
//   1. off() places the chunks of a 64-row tile at distinct 16-byte positions inside the tile, and
//      locate() is its inverse (so the direct-to-LDS loads fill exactly what the reads expect);
//   2. a row-wise 16-byte read of 16 consecutive rows at one chunk touches each of the 64 banks once;
//   3. each half (32 lanes) of a transposing read touches no bank with two different addresses;
//   4. off(r + 16, c) = off(r, c) + 16 * ROWB, which the kernels rely on when they add row-block offsets.
// It also checks that the workgroup-id -> (work item, head) map of the kernels hits every pair exactly once.
#include <cstdio>
#include <map>
#include <set>

#include "../paper_2605_08962_amd/csrc/va_device.h"

template <int D>
static int check() {
    using T = va::LdsTile<D>;
    int bad = 0;
    const int chunks = D / 8, db_n = (D + 31) / 32;
    std::set<int> seen;
    for (int r = 0; r < 64; ++r)
        for (int c = 0; c < chunks; ++c) {
            const int o = T::off(r, c);
            if (o < 0 || o + 16 > 64 * T::ROWB || (o & 15) || !seen.insert(o).second) { ++bad; std::printf("D=%d: off(%d,%d)=%d\n", D, r, c, o); }
            if (r < 48 && T::off(r + 16, c) != o + 16 * T::ROWB) { ++bad; std::printf("D=%d: period at (%d,%d)\n", D, r, c); }
            int rr = -1, cc = -1;
            const int p = (o % (16 * T::ROWB)) / 16;  // position inside the 16-row block
            if (!T::locate(p, rr, cc) || rr != (r & 15) || cc != c) { ++bad; std::printf("D=%d: locate(%d) != (%d,%d)\n", D, p, r & 15, c); }
        }
    int data_positions = 0;
    for (int p = 0; p < T::BLOCK_POS; ++p) { int r, c; if (T::locate(p, r, c)) ++data_positions; }
    if (data_positions != 16 * chunks) { ++bad; std::printf("D=%d: %d data positions\n", D, data_positions); }
    for (int r0 = 0; r0 < 64; r0 += 16)
        for (int c = 0; c < chunks; ++c) {
            std::set<int> banks;
            for (int r = r0; r < r0 + 16; ++r)
                for (int w = 0; w < 4; ++w) banks.insert((T::off(r, c) / 4 + w) % 64);
            if (banks.size() != 64) { ++bad; std::printf("D=%d: row-wise read rows %d.. chunk %d covers %zu banks\n", D, r0, c, banks.size()); }
        }
    for (int row0 = 0; row0 < 16; row0 += 8)
        for (int db = 0; db < db_n; ++db)
            for (int half = 0; half < 2; ++half) {
                std::map<int, std::set<int>> bank_words;
                for (int lane = 32 * half; lane < 32 * half + 32; ++lane) {
                    const int o = T::tr_off(lane, row0, db);
                    if (o < 0 || o + 8 > 64 * T::ROWB) { ++bad; std::printf("D=%d: tr_off out of the tile\n", D); }
                    for (int w = 0; w < 2; ++w) bank_words[(o / 4 + w) % 64].insert(o / 4 + w);
                }
                for (auto& kv : bank_words)
                    if (kv.second.size() != 1) { ++bad; std::printf("D=%d: transposing read row0=%d db=%d half=%d: bank %d conflict\n", D, row0, db, half, kv.first); }
            }
    return bad;
}

static int check_work_order() {
    const int shapes[][3] = {{908, 16, 16}, {1, 16, 16}, {128, 32, 8}, {300, 32, 8}, {257, 8, 8}, {129, 64, 16},
                             {5, 6, 3}, {1000, 24, 8}, {127, 16, 16}, {256, 8, 8}};
    int bad = 0;
    for (auto& sh : shapes) {
        const int n = sh[0], heads = sh[1], kv = sh[2];
        for (int chunk : {1, va::kXcdChunk}) {
            std::set<std::pair<int, int>> seen;
            for (unsigned bid = 0; bid < (unsigned)(n * heads); ++bid) {
                int item, hp;
                va::xcd_item_head(bid, n, heads, kv, chunk, item, hp);
                if (item < 0 || item >= n || hp < 0 || hp >= heads || !seen.insert({item, hp}).second) ++bad;
                // chunked order: the kv head stays on its XCD; item-major order: the slots of item i are those
                // rotated by i, so that every XCD meets every head
                const int slot = chunk == 1 ? ((hp - item) % heads + heads) % heads : hp;
                if (kv % 8 == 0 && (slot % kv) % 8 != (int)(bid % 8)) ++bad;
            }
            if (bad) std::printf("work order n=%d heads=%d kv=%d chunk=%d: %d errors\n", n, heads, kv, chunk, bad);
        }
    }
    return bad;
}

int main() {
    const int bad = check<64>() + check<80>() + check<96>() + check<128>() + check_work_order();
    std::printf(bad ? "FAILED: %d\n" : "lds layouts ok\n", bad);
    return bad != 0;
}
