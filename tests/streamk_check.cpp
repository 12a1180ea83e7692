// Brute-force check of the tiled GEMM's run arithmetic (sk_decomp.h), compiled for the host by test_host_streamk.py.
// For every (B, R, KP) it walks every block's run exactly as the kernel's loop does and checks that the runs tile the
// tail's K ranges without gap or overlap, that no run is empty or shorter than intended, that the closed forms for
// the blocks sharing a tile agree with what the walk found, and that parked pieces never share a slot.
#include <cstdio>
#include <map>
#include <set>
#include <vector>

#include "sk_decomp.h"

using namespace ps;

struct Piece { int lb, kp0, kp1; };

static int check(int B, int R, int KP) {
    const int Bt = sk_tail_blocks(B, R, KP);
    if (Bt < R || Bt > B || (long)Bt > (long)R * KP) { printf("Bt out of range B=%d R=%d KP=%d Bt=%d\n", B, R, KP, Bt); return 1; }
    std::map<int, std::vector<Piece>> by_tile;
    std::set<int> slots;
    for (int lb = 0; lb < B; lb++) {
        int it = lb < Bt ? sk_run_begin(lb, Bt, R, KP) : 0;
        const int it_end = lb < Bt ? sk_run_begin(lb + 1, Bt, R, KP) : 0;
        if (lb < Bt && it >= it_end) { printf("empty run B=%d R=%d KP=%d lb=%d\n", B, R, KP, lb); return 1; }
        int pieces = 0;
        while (it < it_end) {   // the kernel's loop
            const int rt = it / KP;
            const int kp0 = it - rt * KP;
            const int kp1 = (it_end - rt * KP) < KP ? (it_end - rt * KP) : KP;
            it = rt * KP + kp1;
            by_tile[rt].push_back(Piece{lb, kp0, kp1});
            if (!(kp0 == 0 && kp1 == KP)) {   // parked
                const int s = sk_slot(lb, rt);
                if (s < 0 || s >= sk_slots(Bt, R) || !slots.insert(s).second) { printf("slot clash B=%d R=%d KP=%d lb=%d rt=%d\n", B, R, KP, lb, rt); return 1; }
            }
            if (++pieces > 2 && KP > 1) { printf("more than two pieces B=%d R=%d KP=%d lb=%d\n", B, R, KP, lb); return 1; }
        }
    }
    for (int rt = 0; rt < R; rt++) {
        const std::vector<Piece>& v = by_tile[rt];
        if (v.empty()) { printf("tile without a run B=%d R=%d KP=%d rt=%d\n", B, R, KP, rt); return 1; }
        int at = 0;
        for (size_t i = 0; i < v.size(); i++) {
            if (v[i].kp0 != at || v[i].kp1 <= v[i].kp0 || (i && v[i].lb != v[i - 1].lb + 1)) { printf("gap or overlap B=%d R=%d KP=%d rt=%d\n", B, R, KP, rt); return 1; }
            at = v[i].kp1;
        }
        if (at != KP) { printf("K range not covered B=%d R=%d KP=%d rt=%d\n", B, R, KP, rt); return 1; }
        if (sk_first_block(rt, Bt, R, KP) != v.front().lb || sk_last_block(rt, Bt, R, KP) != v.back().lb) {
            printf("closed form off B=%d R=%d KP=%d rt=%d: %d..%d vs %d..%d\n", B, R, KP, rt, sk_first_block(rt, Bt, R, KP), sk_last_block(rt, Bt, R, KP), v.front().lb, v.back().lb);
            return 1;
        }
    }
    return 0;
}

int main() {
    const int kps[] = {1, 2, 3, 4, 5, 8, 11, 16, 17, 32, 64, 128, 224, 448, 1000};
    long n = 0;
    for (int B : {2, 7, 32, 64})
        for (int R = 1; R < B; R++)
            for (int KP : kps) {
                if (check(B, R, KP)) return 1;
                n++;
            }
    printf("OK %ld\n", n);
    return 0;
}
