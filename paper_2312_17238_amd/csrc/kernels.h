// gfx950 device code of the decode step.
#pragma once
#include "kernels_common.h"
#include "kernels_gate.h"
#include "kernels_gemv.h"
#include "kernels_fused.h"
#include "kernels_mfma.h"
#include "kernels_mfma_stream.h"
#include "kernels_mfma16.h"
