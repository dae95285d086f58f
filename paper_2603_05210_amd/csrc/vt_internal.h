// Host-side plan of one vt_draft_head call and the launchers of the kernel families.
// Everything here is internal to the library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace vt {

// Streaming regime (rows <= kGemvMaxRows): workgroups of kGemvThreads threads, each wave
// streams groups of J consecutive W_sub rows.
constexpr int kGemvMaxRows = 16;
constexpr int kGemvThreads = 1024;
constexpr int kGemvWaves = kGemvThreads / 64;
constexpr int kGemvMaxRowsPerBlock = 512;  // W_sub rows one workgroup may own (8 logits per lane at the end)
constexpr int kGemvTargetBlocks = 256;     // one workgroup per compute unit of an MI355X
constexpr int kGemvLdsLimit = 160 * 1024;
constexpr int kMergeThreads = 256;

struct Plan {
    int regime;  // 0 streaming dot product, 1 MFMA GEMM
    int rows, H, Vd, k;
    int KP;      // list length carried in the kernels: k rounded up to a power of two
    // streaming regime
    int NR;      // rows rounded up to a power of two
    int J;       // W_sub rows a wave reduces together
    int rpb;     // W_sub rows per workgroup
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

struct HeadArgs {
    const uint16_t* h;
    const uint16_t* W;
    const int32_t* d2t;
    int32_t* out_ids;
    float* out_logp;
    float* part_val;   // [rows][P][KP]
    int32_t* part_idx; // [rows][P][KP]
    float2* part_stat; // [rows][P]  (max, sum exp(z - max))
    float* logits_out; // optional [rows][Vd]
    float* lse_out;    // optional [rows]
};

struct GemmArgs {
    const void* h;
    const void* W;
    int rows, nchunk, Vd, P;
    int n_vtiles, n_rtiles;
    float* part_val;
    int32_t* part_idx;
    float2* part_stat;
    float* logits_out;
};

#define VT_DECL_GEMM_KP(N) hipError_t launch_gemm_kp##N(const Plan& p, const GemmArgs& ga, hipStream_t s);
VT_DECL_GEMM_KP(1)
VT_DECL_GEMM_KP(2)
VT_DECL_GEMM_KP(4)
VT_DECL_GEMM_KP(8)
VT_DECL_GEMM_KP(16)
VT_DECL_GEMM_KP(32)
VT_DECL_GEMM_KP(64)
#undef VT_DECL_GEMM_KP

hipError_t launch_gemv(const Plan& p, const HeadArgs& a, hipStream_t s);
hipError_t launch_gemm(const Plan& p, const HeadArgs& a, hipStream_t s);
hipError_t launch_merge(const Plan& p, const HeadArgs& a, hipStream_t s);
hipError_t launch_check_ids(const int32_t* ids, int Vd, int V, uint32_t* bitmap, int* err, hipStream_t s);
hipError_t launch_gather(const uint16_t* W, int H, const int32_t* ids, int Vd, uint16_t* W_sub, int32_t* d2t,
                         hipStream_t s);

// GEMM tile shapes (vocab x rows per workgroup) and their partial counts; defined with the kernel.
int gemm_pick_tile(int rows, int H, int Vd, int KP);
void gemm_tile_dims(int tile, int& BMV, int& BNR, int& parts_per_vtile);

}  // namespace vt
