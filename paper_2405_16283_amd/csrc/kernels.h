// Interface between the executor (host) and the gfx950 task kernels.
//
// Every kernel is *grouped*: one launch serves a batch of ready memgraph vertices of the same
// launch class.  Because a memgraph fixes the GPU location of every tensor before execution
// (Section 5, first paragraph), the per-vertex operand tables can be built once, at executor
// creation, and stay in device memory; a launch only names the vertices it covers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "turnip.h"

namespace tn {

// One kernel-call vertex, as the kernels see it.
struct OpDesc {
  void* out;        // device address of the output tensor
  uint32_t ptr0;    // index of the first operand address in the pointer table
  uint32_t aux0;    // index of the first auxiliary integer (meaning depends on the kind)
  int32_t rows, cols;  // output shape
  int32_t n_in;
  int32_t nblocks;  // workgroups this vertex needs in its launch class
  int32_t dtype;    // storage type of its non-statistics operands (TN_F32 / TN_BF16)
  int32_t trans_b;  // gemm: B tiles are stored [cols, K]
  tn_op_params p;
};

// Launch classes: vertices of one class can share a launch.
enum LaunchClass {
  LC_GEMM_F32 = 0,   // generic fp32-accumulate GEMM on the vector ALUs, any layout, fp32 or bf16 storage
  LC_GEMM_BF16_NT,   // MFMA bf16 GEMM, B tiles stored [cols, K], 128x128 tile per workgroup
  LC_GEMM_BF16_NT256,  // the same for output tiles of at least 256x256: 256x256 per workgroup
  LC_RMS_STAT,
  LC_RMS_APPLY,
  LC_ROPE,
  LC_ATTN_F32,       // attention block on the vector ALUs (fp32 storage, or shapes the MFMA kernel does not take)
  LC_ATTN_BF16,      // MFMA attention block
  LC_ATTN_COMBINE,
  LC_SILU_MUL,
  LC_ADD,
  LC_SILU_BWD,
  LC_RMS_BWD_STAT,
  LC_RMS_BWD_APPLY,
  LC_ATTN_BWD,       // attention backward on the vector ALUs (statistics, dQ, dK, dV)
  LC_ATTN_BWD_BF16,  // MFMA attention backward: statistics; the next three values are its dQ, dK and dV forms
  LC_ATTN_BWD_BF16_DQ,
  LC_ATTN_BWD_BF16_DK,
  LC_ATTN_BWD_BF16_DV,
  LC_TRANSPOSE,
  LC_ZERO,           // clears a tensor: the start of a sum's output
  LC_SOFTMAX_STAT,   // row maximum and sum of exponentials over the score tiles of a row block
  LC_SOFTMAX_APPLY,  // probabilities of one score tile
  LC_COUNT,
  // Not a class of its own for grouping: the form in which a group of LC_GEMM_BF16_NT256 vertices is
  // launched when it has too few 256x256 tiles to give every CU one (128x128 tiles, same bits).
  LC_GEMM_BF16_NT256_SMALL
};

// Vertices per launch.  The list travels in the kernel arguments (4 KiB at most), as 16-bit
// offsets from the smallest descriptor index of the group.
constexpr int kMaxBatch = 1920;
constexpr uint32_t kMaxBatchSpan = 65535;  // largest descriptor index distance inside one group

struct Batch {
  int32_t n;
  uint32_t base;            // smallest descriptor index of the group
  uint16_t idx[kMaxBatch];  // descriptor index minus base
  __host__ __device__ uint32_t at(uint32_t i) const { return base + idx[i]; }
};

struct DeviceTables {
  const OpDesc* descs;
  void* const* ptrs;
  const int32_t* aux;
  const double* rope_theta;  // base^(-2i/head_dim), i < head_dim/2, for the graph's rotary vertices
};

// A group of tensor copies between GPU memory and pinned (device-visible) host memory, moved by
// one kernel launch: offloads, reloads, loads and stores of the memgraph.  The copy routine of
// the runtime spends a launch and a gap per tensor, which at tile sizes of a few hundred KiB
// leaves half of the host link idle.
constexpr int kMaxCopies = 128;
constexpr int kCopyThreads = 1024;
constexpr int kCopyLoads = 2;  // 16-byte loads in flight per lane
constexpr uint32_t kCopyBlockBytes = kCopyLoads * 16 * kCopyThreads;  // bytes one workgroup moves per step: 32 KiB
constexpr int kDefaultCopyWorkgroups = 8;
constexpr int kDeviceCopyWorkgroups = 512;  // copies that stay inside GPU memory: two per compute unit
struct CopyItem {
  const void* src;
  void* dst;
  uint32_t bytes;
  uint32_t first_block;  // index of its first 32 KiB piece among the pieces of the group
};
struct CopyBatch {
  int32_t n;
  int32_t total_blocks;
  CopyItem it[kMaxCopies];
};
// max_workgroups <= 0 selects kDefaultCopyWorkgroups
hipError_t launch_copies(const CopyBatch& b, int max_workgroups, hipStream_t stream);

// A region of GPU memory that exists from the moment the library is loaded until the process ends,
// for callers that want the operand tables of a run somewhere nobody has to allocate.  Each GPU
// holds its own copy of the region at its own address; *ptr receives the address on the current
// device (looked up once per device).  Contents are whatever the last user left there.
constexpr size_t kStaticTableBytes = 8u << 20;
hipError_t static_table_region(void** ptr);

// Workgroups a vertex needs in the given class (host side, used to fill OpDesc::nblocks).
int32_t blocks_for(int cls, const OpDesc& d, const int32_t* aux);

// Enqueues one grouped launch on `stream`.  All vertices of the batch share the class, the storage
// type and (for attention) the head size.  max_blocks = largest nblocks in the batch.
hipError_t launch_batch(int cls, int dtype, int head_dim, const DeviceTables& t, const Batch& b,
                        int32_t max_blocks, hipStream_t stream);

}  // namespace tn
