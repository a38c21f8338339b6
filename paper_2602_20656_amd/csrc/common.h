// Internal helpers shared by the translation units of liblagom (not part of the ABI).
#pragma once
#include <cstdarg>
#include <cstdint>
#include "lagom.h"

namespace lagom {

// Records the calling thread's error text and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline int elem_size(int dtype) { return dtype == LAGOM_F32 ? 4 : (dtype == LAGOM_BF16 ? 2 : 0); }

// Argument checks shared by lagom_comm_kernel and the overlap runner.
int check_cfg(const lagom_cfg* cfg);
int check_comm_args(int op, int dtype, const void* const* srcs, int nsrc, void* const* dsts, int ndst,
                    int64_t count);
int check_comm_steps(int dtype, const lagom_comm_step* steps, int nsteps, int64_t count);
int check_gemm_args(const void* A, const void* B, const void* C, int64_t M, int64_t N, int64_t K, int out_dt);

}  // namespace lagom
