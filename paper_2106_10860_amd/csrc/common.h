// Internal declarations shared by the translation units of libmaddness.
// Nothing here is part of the public ABI (see include/maddness.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "maddness.h"

namespace maddness {

// Records a message for maddness_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);

// Records which kernel a call selected, for maddness_last_kernel(): `family` is the
// kernel's name, `instance` the launcher's __PRETTY_FUNCTION__ (its "[...]" part lists the
// template arguments) or nullptr.  The first kernel noted in a call is the one kept.
void note_kernel(const char *family, const char *instance);

// Turns a hipError_t into MADDNESS_E_HIP (with message) or MADDNESS_OK.
int check_hip(hipError_t e, const char *what);

// Properties of the current device, queried once per process.
struct DeviceInfo {
    int cus;            // compute units
    int lds_per_block;  // bytes of LDS one workgroup may use
};
const DeviceInfo &device_info();

// Dynamic LDS beyond the default 64 KiB has to be granted per kernel.  Done once
// per kernel and process (the library drives one device per process); the status
// of that one call is returned every time.
template <auto Kernel>
int allow_full_lds()
{
    static std::once_flag once;
    static int status = MADDNESS_OK;
    std::call_once(once, [] {
        status = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               device_info().lds_per_block),
                           "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
    });
    return status;
}

// The input matrix A of the encoders: element type (a maddness_dtype), storage
// order and leading dimension in elements (row stride when stored by rows, column
// stride when stored by columns).
struct MatrixA {
    const void *data = nullptr;
    int dtype = MADDNESS_F32;
    bool col_major = false;
    int64_t ld = 0;
    bool plain() const { return dtype == MADDNESS_F32 && !col_major; }
    int64_t row_stride() const { return col_major ? 1 : ld; }
    int64_t col_stride() const { return col_major ? ld : 1; }
    int elem_bytes() const { return dtype == MADDNESS_F32 ? 4 : (dtype == MADDNESS_U8 ? 1 : 2); }
};

// Encode only: A -> packed codes.
int launch_encode(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                  hipStream_t stream);

// Scan (A == nullptr: codes_in is read) or fused encode+scan (A != nullptr:
// codes are computed, and also written to codes_out when it is not null).
// averaged: the table entries are aggregated by pairwise averages in blocks of 16
// codebooks (Appendix D) instead of the exact sum; C must be a multiple of 16.
int launch_scan(const maddness_params *p, const MatrixA *A, const uint8_t *codes_in,
                int32_t C, int32_t M, int64_t N, const uint8_t *luts, const float *scale,
                const float *offset, float *out, int64_t ldo, uint16_t *acc, uint8_t *codes_out,
                bool averaged, hipStream_t stream);

// Row-streaming kernels specialised for C in {16, 32, 64}, rows of 16-byte pieces
// and (fused, scan) one tile of <= 256 output columns whose tables fit in LDS, or
// column tiles for larger tables.  launch_fused_rows hands the shapes the matrix-core
// kernel is better at over to it.
// Each returns MADDNESS_OK after a launch, 1 if the shape is not covered (nothing
// was launched; the caller falls back to the general kernels), or an error status.
int launch_encode_rows(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                       hipStream_t stream);
int launch_scan_rows(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                     const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                     bool averaged, hipStream_t stream);
int launch_fused_rows(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M,
                      const uint8_t *luts, const float *scale, const float *offset, float *out,
                      int64_t ldo, uint16_t *acc, uint8_t *codes, bool averaged, hipStream_t stream);

// Current value of a maddness_option (maddness_set_option; 0 = the library chooses).
int32_t option(int which);
// MADDNESS_OPT_KERNELS >= 1: the scan stays off the matrix cores (the vector-ALU kernels
// stay testable and comparable).
bool vector_scan_only();

// The exact scan on the matrix cores (one-hot codes x tables, int8 MFMA): C a multiple
// of 8 up to 64, many rows.  Same return convention as the row kernels.
int launch_scan_mfma(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                     const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                     hipStream_t stream);

// Fused encode + exact scan in phases with the scan on the matrix cores (C = 32 or 64,
// many rows; A row-major of any element type, or stored by columns with N a multiple
// of 4; C = 16 with row-major fp32 A).  The callers use it for many rows: where the one-kernel-per-wavefront designs
// are bound by the vector ALUs (tables larger than LDS, narrow element types, A stored by
// columns), and for C = 16 and 32 in general, because whole-chip read and write phases suit HBM.
int launch_fused_mfma(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M, const uint8_t *luts,
                      const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                      uint8_t *codes, hipStream_t stream);

// Encode only with the first phase of that kernel (row-major fp32 A, C = 16, 32 or 64, many rows).
int launch_encode_phased(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                         hipStream_t stream);

// A stored by columns (any element type): only the four split columns of every
// codebook are read.  Same return convention as the row kernels.
int launch_encode_cols(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                       hipStream_t stream);
int launch_fused_cols(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M,
                      const uint8_t *luts, const float *scale, const float *offset, float *out,
                      int64_t ldo, uint16_t *acc, uint8_t *codes, bool averaged, hipStream_t stream);

size_t build_luts_workspace_bytes(int32_t D, int32_t C, int32_t M);
// pooled: Appendix A as printed (one scale, one offset per codebook) instead of
// per-column scale and offsets.
int launch_build_luts(const maddness_params &p, const float *B, int32_t M, int64_t ldb,
                      uint8_t *luts, float *scale, float *offset, void *workspace, bool pooled,
                      hipStream_t stream);

// The learning step (Section 4.2-4.3; Appendix C).  bounds_host: [C][2] first and one-past-last
// column of every codebook, in host memory; dmax: the widest subspace.
size_t learn_trees_workspace_bytes(int64_t N, int32_t C, int32_t dmax);
size_t learn_prototypes_workspace_bytes(int32_t D, int32_t C);
int learn_max_subspace_width();
int launch_learn_trees(const float *A, int64_t N, int64_t lda, int32_t C, const int32_t *bounds_host, int32_t dmax,
                       int32_t *split_dims, float *thresholds, uint8_t *codes, void *workspace, hipStream_t stream);
int launch_learn_prototypes(const uint8_t *codes, const float *A, int64_t N, int64_t lda, int32_t D, int32_t C,
                            const int32_t *bounds_host, bool ridge, double lambda, float *prototypes, void *workspace,
                            hipStream_t stream);

// Device address of the library's own table-build workspace (MADDNESS_STATIC_WORKSPACE_BYTES,
// one per GPU) on the current device.  Allocates nothing.
int static_workspace(void **workspace);

}  // namespace maddness
