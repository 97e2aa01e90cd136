// Host side of the C ABI without a GPU: table builder and argument checks; built with the host
// sanitizers by tests/test_host_sanitizers.py.
#include "terngrad.h"
#include <cstdio>
#include <vector>
int main() {
    std::vector<int64_t> off = {0, 5, 5, 1030, 1031, 50000, 50000, 70001};
    int64_t te, nt, ce, ns;
    if (tg_describe_tables((int64_t)off.size() - 1, off.data(), 4, &te, &nt, nullptr, nullptr, 0, &ce, &ns, nullptr, 0) != TG_OK) return 1;
    std::vector<int32_t> tl(nt); std::vector<uint8_t> tw(nt); std::vector<int64_t> seg(3 * ns);
    if (tg_describe_tables((int64_t)off.size() - 1, off.data(), 4, &te, &nt, tl.data(), tw.data(), nt, &ce, &ns, seg.data(), ns) != TG_OK) return 2;
    int64_t bad[3] = {0, 5, 3};
    if (tg_describe_tables(2, bad, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, nullptr, 0) != TG_ERR_INVALID_ARG) return 3;
    tg_plan* p = nullptr;
    if (tg_plan_create(2, bad, 1, &p) != TG_ERR_INVALID_ARG) return 4;
    if (tg_clip_stats(nullptr, 1, nullptr, 2.5f, nullptr, nullptr, nullptr) != TG_ERR_INVALID_ARG) return 5;
    if (tg_average_float(1, 4, nullptr, nullptr, nullptr) != TG_ERR_INVALID_ARG) return 6;
    std::printf("ok tiles=%lld segs=%lld %s\n", (long long)nt, (long long)ns, tg_strerror(TG_ERR_ALIGNMENT));
    return 0;
}
