// The host-side plan of one vt_draft_head call: which kernel family serves a shape, how the
// vocabulary is cut into workgroups and tiles, how many partial results a row gets and where
// they live in the caller's workspace.  Plain C++ with no HIP dependency: the argument
// validators use it too, and a host-sanitizer build compiles it on its own.
#pragma once

#include <stddef.h>
#include <stdint.h>

namespace vt {

// Streaming regime (rows <= kGemvMaxRows): workgroups of kGemvThreads threads, each wave
// streams groups of J consecutive W_sub rows.
constexpr int kGemvMaxRows = 16;
constexpr int kFewMaxRows = 64;  // the kernel for a few rows: up to four groups of 16 rows share the W_sub stream
// three or four groups only over a narrow vocabulary (measured at H = 4096, 48 / 64 rows: 44 / 46 us
// against the GEMM regime's 57 at V_draft = 13264, 88 / 94 against 85 at 32768)
constexpr int kFewWideMaxVd = 16384;
constexpr int kFewOneRowMinVd = 8192;  // one MXFP4 row goes to that kernel from this vocabulary size on
constexpr int kGemvThreads = 1024;
constexpr int kGemvWaves = kGemvThreads / 64;
constexpr int kGemvMaxRowsPerBlock = 512;  // W_sub rows one workgroup may own (8 logits per lane at the end)
constexpr int kGemvTargetBlocks = 256;     // one workgroup per compute unit of an MI355X
// dynamic LDS a streaming kernel may ask for: the 160 KiB of a compute unit less the few bytes of
// static LDS the kernels declare themselves
constexpr int kGemvLdsLimit = 160 * 1024 - 256;
// The caller's workspace starts with a header of this many bytes: the arrival counters of the
// single-launch merge, one per 256 bytes so that no two share a cache line (counter 0: the call;
// counters 1..16: groups of 16 workgroups).  All zero between calls: vt_draft_head_workspace_init
// zeroes them once, and whoever sees a counter full puts it back to zero.
constexpr size_t kWorkspaceHeader = 8192;  // = VT_WORKSPACE_HEADER_BYTES of the C header
constexpr int kArriveStrideWords = 64;
constexpr int kMergeThreads = 256;

struct Plan {
    int regime;  // 0 streaming dot product, 1 MFMA GEMM
    int rows, H, Vd, k;
    int KP;      // list length carried in the kernels: k rounded up to a power of two
    // streaming regime
    int NR;      // rows rounded up to a power of two
    int J;       // W_sub rows a wave reduces together
    int rpb;     // W_sub rows per workgroup
    int one_row; // the dedicated one-row kernel (H = 512, 1024, 2048 or 4096, lists of at most 16)
    int few_rows; // the dedicated kernel for 2..kFewMaxRows rows (H = 2048 or 4096, lists of at most 16)
    int nsg;     // its groups of 16 rows, each served by blocks / nsg workgroups
    int fused;   // the streaming kernel's last workgroup also does the final merge
    int mfma;    // matrix-core variant of the streaming kernel (several rows, H % 256 == 0)
    int ks;      // its slices of the hidden dimension per 16-row group (narrow ranges: keeps 16 waves busy)
    // GEMM regime
    int tile;    // index into the table of tile shapes
    int n_vtiles, n_rtiles;
    // both
    int blocks;  // workgroups of the projection kernel
    int P;       // partial results per row handed to the merge kernel
    size_t off_val, off_idx, off_stat, total_bytes;
};

// Fills `p`; returns false when the shape is not servable (caller has validated ranges).
bool make_plan(int64_t rows, int64_t H, int64_t Vd, int k, Plan& p);

// The plan of a draft step over a compressed W_sub (format codes as in the C header); false when
// the shape is not served.
bool make_plan_q(int fmt, int64_t rows, int64_t H, int64_t Vd, int k, Plan& p);

// GEMM tile shapes (vocab x rows per workgroup) and their partial counts.
int gemm_pick_tile(int rows, int H, int Vd, int KP);
void gemm_tile_dims(int tile, int& BMV, int& BNR, int& parts_per_vtile);

}  // namespace vt
