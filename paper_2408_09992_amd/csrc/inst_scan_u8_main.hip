// Instantiates one group of catalogue-scan kernels (see the instance lists in kernels.hpp).
#define PQ_INSTANCE_TU
#include "kernels.hpp"
namespace pqk {
PQ_SCAN_INSTANCES_U8_MAIN(PQ_SCAN_DEFINE)
PQ_SCAN_INSTANCES_STAMPED(PQ_SCAN_DEFINE6)
}
