// Sizes shared by the workspace carving and the backward kernels' launchers.
#pragma once
#define SPK_NORM_BWD_BLOCKS 256   // partial rows of the gain-gradient reduction
#define SPK_MSE_PARTS 1024        // partial sums of the loss reduction
#define SPK_STATIC_MAX_D 4096      // widest row spk_rmsnorm_bwd_static's built-in partial-row array holds
#define SPK_SPIN_MAX_US 20000        // longest delay one spin kernel may take (debug delay mode)
// decode attention keeps one fp32 score per cached position in LDS
constexpr int kDecodeMaxLen = 32768;
constexpr size_t kDecodeMaxLds = ((size_t)kDecodeMaxLen + 128 + 8 + 4 * 512 + 2048) * 4;
