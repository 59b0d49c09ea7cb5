// Kernel instantiations for one cell / storage type (compiled separately to
// keep build times short).
#include "cells.h"
#include "pararnn/launch_impl.h"
namespace pararnn { template struct Kernels<LstmDiag, float>; }
