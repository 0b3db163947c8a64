// CPU check of the parser of the SCORCH_SPMM_TUNE text: values, defaults, malformed items, and that it is
// re-entrant (eight threads parse different texts at once, ten thousand times each, and always get their own answer).
// Prints "ok" or the first failure.
#include <cstdio>
#include <string>
#include <thread>
#include <vector>

#include "tuning.h"

using namespace scorch;

#define EXPECT(cond)                                             \
    do {                                                         \
        if (!(cond)) {                                           \
            std::printf("line %d: %s\n", __LINE__, #cond);       \
            return 1;                                            \
        }                                                        \
    } while (0)

int main() {
    Tuning d = parse_tuning(nullptr);
    EXPECT(d.bn == 0 && d.alpha == 0 && d.lw == 0 && d.ch == 0 && d.bch == 0 && d.u == 0);
    EXPECT(d.nt == -1 && d.sliced == -1 && d.pack == -1 && d.panel == -1 && d.hot == -1 && d.sdblk == -1 && d.fix == -1 && d.cold == 0);
    Tuning e = parse_tuning("");
    EXPECT(e.bn == 0 && e.sdblk == -1);
    Tuning t = parse_tuning("bn=64,alpha=2,lw=8,ch=32,bch=64,u=4,nt=0,sliced=64,pack=1,panel=2,hot=65536,sdblk=3,fix=1,cold=2");
    EXPECT(t.bn == 64 && t.alpha == 2 && t.lw == 8 && t.ch == 32 && t.bch == 64 && t.u == 4 && t.nt == 0);
    EXPECT(t.sliced == 64 && t.pack == 1 && t.panel == 2 && t.hot == 65536 && t.sdblk == 3 && t.fix == 1 && t.cold == 2);
    t = parse_tuning(" bn = 128 ,, lw=0,junk,=5,bnx=3,b=9,ch=12x,hot=-1,sdblk=+2,panel=,alpha=99999999999,u=8,");
    EXPECT(t.bn == 128 && t.lw == 0 && t.ch == 0 && t.hot == -1 && t.sdblk == 2 && t.panel == -1 && t.u == 8);
    EXPECT(t.alpha == 0x7fffffff);
    t = parse_tuning("bn=16,bn=32");  // the last one wins
    EXPECT(t.bn == 32);
    t = parse_tuning("sdblk=0");
    EXPECT(t.sdblk == 0 && t.bn == 0);
    std::string longtext;
    for (int i = 0; i < 2000; ++i) longtext += "zz=1,";
    longtext += "lw=7";
    EXPECT(parse_tuning(longtext.c_str()).lw == 7);  // no fixed-size copy of the text

    std::vector<std::thread> th;
    std::vector<int> bad(8, 0);
    for (int w = 0; w < 8; ++w)
        th.emplace_back([w, &bad] {
            const std::string text = "bn=" + std::to_string(16 + w) + ",lw=" + std::to_string(w) + ",sdblk=" + std::to_string(w % 3);
            for (int i = 0; i < 10000; ++i) {
                const Tuning x = parse_tuning(text.c_str());
                if (x.bn != 16 + w || x.lw != w || x.sdblk != w % 3) bad[w] = 1;
            }
        });
    for (auto &x : th) x.join();
    for (int w = 0; w < 8; ++w) EXPECT(!bad[w]);
    std::printf("ok\n");
    return 0;
}
