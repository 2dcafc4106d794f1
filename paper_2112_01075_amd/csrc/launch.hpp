// Host-callable launchers of the gfx950 kernels (defined in kernels.hip).
#pragma once
#include <cstddef>
#include <cstdint>

#include "copyop.hpp"

namespace redist {

constexpr int kMaxExecDevices = 128;

// Shard pointers travel as kernel arguments: no device-side table to keep in sync per call.  Meshes
// with more than kMaxExecDevices devices pass `ext`, a device-memory array of all shard pointers,
// instead (p[] is then unused).
struct PtrTable {
  void* p[kMaxExecDevices];
  void* const* ext;  // host side only: selects the kernel variant that reads PtrTableExt
#if defined(__HIPCC__)
  __device__ __forceinline__ void* at(int i) const { return p[i]; }
#endif
};
// The kernel-side view for big meshes.  A separate type (and kernel instantiation) rather than a
// run-time choice inside at(): the choice would sit on the dependent chain in front of a workgroup's
// first load (measured: 9 % on the headline workload).
struct PtrTableExt {
  void* const* ext;
#if defined(__HIPCC__)
  // (constant address space: the table is written before the launch and read with scalar loads)
  __device__ __forceinline__ void* at(int i) const {
    typedef void* const __attribute__((address_space(4))) * table_ptr;
    return ((table_ptr)(uintptr_t)ext)[i];
  }
#endif
};

// Enqueue one copy op; dev_boxes / dev_dst_list are the device copies of op.boxes / op.dst_list.
// Returns the hipError_t of the launch as int (0 = success).
int launch_copy_op(const CopyOp& op, const void* dev_boxes, const void* dev_dst_list, const PtrTable& src,
                   const PtrTable& dst, void* stream);
// Same for a row-complete (LDS-staged) op.
int launch_row_op(int kind, const RowOp& op, const void* dev_boxes, const void* dev_pieces, const void* dev_list,
                  const PtrTable& src, const PtrTable& dst, void* stream);
// Same for a cell-complete op (meshes whose shard pointers travel as kernel arguments only).
int launch_cell_op(int kind, const CellOp& op, const void* dev_boxes, const void* dev_list, const PtrTable& src,
                   const PtrTable& dst, void* stream);
// Device-side pointer tables of meshes beyond kMaxExecDevices, written by small kernels on `stream`:
// dev_out[i] = host_ptrs[i] (the pointers travel as kernel arguments), and dev_out[i] = base + i * stride.
int launch_ptr_table(const void* const* host_ptrs, int n, void** dev_out, void* stream);
int launch_ptr_table_strided(void* base, int64_t stride, int n, void** dev_out, void* stream);
int launch_copy_baseline(void* dst, const void* src, int64_t bytes, void* stream);
// The fixed scratch area in the library's device image (one per GPU), for the entry point that allocates nothing:
// its device address on the current device (0 = success, else the hipError_t), and a copy of host memory into
// device memory in which the bytes travel as kernel arguments (no staging buffer, no runtime copy routine).
constexpr size_t kStaticScratchBytes = 32u << 20;
int static_scratch_base(void** out);
int launch_upload(const void* host_src, size_t bytes, void* dev_dst, void* stream);
const char* kernel_name_of(int kind);
const char* row_kernel_name_of(int kind);
const char* cell_kernel_name_of(int kind);

}  // namespace redist
