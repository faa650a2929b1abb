// Instantiates the candidate-list kernels for short lists (see the instance lists in kernels.hpp).
#define PQ_INSTANCE_TU
#include "kernels.hpp"
namespace pqk {
PQ_SUBSET_INSTANCES(PQ_SUBSET_DEFINE)
}
