// Prints what the launch-shape rules of the library decide for the sizes given on the command
// line, so that a test can check them without a GPU.  Links tables.cpp only.
//   launch_rules update <n_workers> <n_cus> <lds_per_cu> <forced> <workgroups>...
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "plan.hpp"

namespace mgwfbp {
void set_error(const std::string &) {}
}  // namespace mgwfbp

int main(int argc, char **argv)
{
    if (argc < 6 || std::strcmp(argv[1], "update") != 0) return 2;
    const int n_workers = std::atoi(argv[2]), n_cus = std::atoi(argv[3]);
    const unsigned lds = static_cast<unsigned>(std::strtoul(argv[4], nullptr, 10));
    const int forced = std::atoi(argv[5]);
    for (int i = 6; i < argc; ++i) {
        const unsigned long long w = std::strtoull(argv[i], nullptr, 10);
        std::printf("%llu %u\n", w, mgwfbp::update_occupancy_lds(n_workers, n_cus, lds, w, forced));
    }
    return 0;
}
