// Instantiation unit of the streaming pass: compiled once per update kind, dtype and range of K
// (-DDYNAMIX_INST_OPT=<0|1|2> -DDYNAMIX_INST_DT=<0|1|2> -DDYNAMIX_INST_LO=<first K>; eight
// consecutive K per unit) so that the kernels build in parallel.
#include "stream_pass.h"

#ifndef DYNAMIX_INST_DT
#error "define DYNAMIX_INST_DT and DYNAMIX_INST_LO"
#endif
#ifndef DYNAMIX_INST_OPT
#define DYNAMIX_INST_OPT 0
#endif

namespace dynamix {

#define DYNAMIX_CAT2(a, b, c, d, e, f) a##b##c##d##e##f
#define DYNAMIX_CAT(a, b, c, d, e, f) DYNAMIX_CAT2(a, b, c, d, e, f)
#define LAUNCH_NAME \
    DYNAMIX_CAT(launch_stream_pass_, DYNAMIX_INST_OPT, _, DYNAMIX_INST_DT, _, DYNAMIX_INST_LO)
#define OCC_NAME \
    DYNAMIX_CAT(occupancy_stream_pass_, DYNAMIX_INST_OPT, _, DYNAMIX_INST_DT, _, DYNAMIX_INST_LO)

hipError_t LAUNCH_NAME(int K, int grid, const StreamArgs& a, hipStream_t s)
{
    constexpr int DT = DYNAMIX_INST_DT, LO = DYNAMIX_INST_LO, OPT = DYNAMIX_INST_OPT;
    switch (K - LO) {
    case 0: return launch_one<DT, LO + 0, OPT>(grid, a, s);
    case 1: return launch_one<DT, LO + 1, OPT>(grid, a, s);
    case 2: return launch_one<DT, LO + 2, OPT>(grid, a, s);
    case 3: return launch_one<DT, LO + 3, OPT>(grid, a, s);
    case 4: return launch_one<DT, LO + 4, OPT>(grid, a, s);
    case 5: return launch_one<DT, LO + 5, OPT>(grid, a, s);
    case 6: return launch_one<DT, LO + 6, OPT>(grid, a, s);
    case 7: return launch_one<DT, LO + 7, OPT>(grid, a, s);
    default: return hipErrorInvalidValue;
    }
}

int OCC_NAME(int K)
{
    constexpr int DT = DYNAMIX_INST_DT, LO = DYNAMIX_INST_LO, OPT = DYNAMIX_INST_OPT;
    switch (K - LO) {
    case 0: return occupancy_one<DT, LO + 0, OPT>();
    case 1: return occupancy_one<DT, LO + 1, OPT>();
    case 2: return occupancy_one<DT, LO + 2, OPT>();
    case 3: return occupancy_one<DT, LO + 3, OPT>();
    case 4: return occupancy_one<DT, LO + 4, OPT>();
    case 5: return occupancy_one<DT, LO + 5, OPT>();
    case 6: return occupancy_one<DT, LO + 6, OPT>();
    case 7: return occupancy_one<DT, LO + 7, OPT>();
    default: return 0;
    }
}

}  // namespace dynamix
