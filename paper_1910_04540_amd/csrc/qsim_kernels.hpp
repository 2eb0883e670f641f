// All kernels of libqsim (hand-written HIP for gfx950); see qsim_kernel_common.hpp for what they share.
#pragma once

#include "qsim_kernel_common.hpp"
#include "qsim_elementwise_kernels.hpp"
#include "qsim_block_register_kernels.hpp"
#include "qsim_block_two_pass_kernels.hpp"
#include "qsim_block_single_pass_kernels.hpp"
#include "qsim_sgd_kernels.hpp"
