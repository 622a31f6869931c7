// All device kernels of the path except the GEMM engine (dn_gemm.h).
#pragma once
#include "dn_common.h"
#include "dn_kernels_dense.h"
#include "dn_kernels_stream.h"
#include "dn_kernels_band.h"
#include "dn_kernels_vector.h"
#include "dn_kernels_part.h"
