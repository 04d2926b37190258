// CPU check of the paged cache's host bookkeeping (paper_2504_07878_amd/csrc/kv_pages.h): random appends, rollbacks,
// forks and restarts over a small pool, with the pages' contents emulated in host arrays. After every operation each slot
// must read back exactly the sequence a plain per-slot vector holds, reference counts must equal the number of table entries
// that name a page, every page is either free or referenced, the predicted demand equals the pages actually taken, and an
// operation that does not fit leaves everything untouched.
#include "../paper_2504_07878_amd/csrc/kv_pages.h"

#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

using tr::KvPages;

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::printf("FAILED line %d: %s\n", __LINE__, #c); if (++fails > 10) std::exit(1); } } while (0)

int main()
{
    const int slots = 6, page = 32, max_seq = 300, maxp = (max_seq + page - 1) / page;
    for (int pool : {slots * maxp, 17}) {
        KvPages P;
        P.init(slots, page, maxp, pool);
        std::vector<std::vector<int>> data((size_t)pool, std::vector<int>((size_t)page, -1));   // what the device pages would hold
        std::vector<std::vector<int>> want((size_t)slots);                                       // the sequences, plainly
        std::mt19937 rng(7878 + pool);
        int next = 0, refused = 0, copied = 0;
        auto write = [&](int s, int from, int to) {   // positions [from, to) of slot s get fresh values
            for (int p = from; p < to; ++p) {
                const int pg = P.row(s)[p / page];
                CHECK(P.refc[(size_t)pg] == 1);       // never write into a shared page
                data[(size_t)pg][(size_t)(p % page)] = next;
                want[(size_t)s].push_back(next++);
            }
        };
        auto grow_many = [&](std::vector<int> sl, std::vector<int> add) {   // one call over several slots, all or nothing
            std::vector<int> from, to;
            for (size_t i = 0; i < sl.size(); ++i) { from.push_back((int)want[(size_t)sl[i]].size()); to.push_back(from.back() + add[i]); }
            const int need = P.demand((int)sl.size(), sl.data(), from.data(), to.data()), free0 = P.free_count();
            if (need > free0) { ++refused; return false; }
            std::vector<KvPages::Copy> copies;
            for (size_t i = 0; i < sl.size(); ++i) P.grow(sl[i], from[i], to[i], copies);
            CHECK(free0 - P.free_count() == need);
            for (const auto &c : copies) { data[(size_t)c.to] = data[(size_t)c.from]; ++copied; }
            for (size_t i = 0; i < sl.size(); ++i) write(sl[i], from[i], to[i]);
            return true;
        };
        for (int step = 0; step < 20000; ++step) {
            const int op = (int)(rng() % 10), s = (int)(rng() % slots);
            if (op < 5) {            // append to one or several distinct slots
                std::vector<int> sl, add;
                const int k = 1 + (int)(rng() % 3);
                for (int i = 0; i < k; ++i) {
                    const int c = (s + i) % slots, room = max_seq - (int)want[(size_t)c].size();
                    if (room <= 0) continue;
                    sl.push_back(c); add.push_back(1 + (int)(rng() % std::min(room, 70)));
                }
                if (!sl.empty()) {
                    const KvPages before = P;
                    if (!grow_many(sl, add)) { CHECK(before.table == P.table && before.refc == P.refc && before.free_ == P.free_ && before.npages == P.npages); }
                }
            } else if (op < 7) {     // roll back
                const int len = (int)want[(size_t)s].size(), to = len ? (int)(rng() % (len + 1)) : 0;
                P.shrink(s, to);
                want[(size_t)s].resize((size_t)to);
            } else if (op < 9) {     // fork
                const int d = (s + 1 + (int)(rng() % (slots - 1))) % slots;
                P.shrink(d, 0);
                P.share(s, d);
                want[(size_t)d] = want[(size_t)s];
            } else {                 // start over with a new prompt; on failure the old sequence must survive
                const KvPages before = P;
                const std::vector<int> old = want[(size_t)s];
                P.shrink(s, 0);
                want[(size_t)s].clear();
                if (!grow_many({s}, {1 + (int)(rng() % 120)})) { P = before; want[(size_t)s] = old; }
            }
            // invariants
            std::vector<int> refs((size_t)pool, 0);
            for (int t = 0; t < slots; ++t) {
                CHECK(P.npages[(size_t)t] == P.pages_for((int)want[(size_t)t].size()));
                for (int k = 0; k < P.npages[(size_t)t]; ++k) refs[(size_t)P.row(t)[k]] += 1;
                for (size_t p = 0; p < want[(size_t)t].size(); ++p)
                    CHECK(data[(size_t)P.row(t)[p / page]][p % page] == want[(size_t)t][p]);
            }
            std::vector<char> is_free((size_t)pool, 0);
            for (int pg : P.free_) { CHECK(!is_free[(size_t)pg]); is_free[(size_t)pg] = 1; }
            for (int pg = 0; pg < pool; ++pg) { CHECK(refs[(size_t)pg] == P.refc[(size_t)pg] || is_free[(size_t)pg]); CHECK((refs[(size_t)pg] == 0) == (is_free[(size_t)pg] != 0)); }
        }
        std::printf("pool %d: %d calls refused, %d pages copied before a write\n", pool, refused, copied);
        if (pool == 17) { CHECK(refused > 0); }
        CHECK(copied > 0);
    }
    std::printf(fails ? "FAILED\n" : "OK\n");
    return fails ? 1 : 0;
}
