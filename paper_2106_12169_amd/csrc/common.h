// Host-side plumbing shared by the C-ABI entry points: status codes, the
// thread-local error text, argument checks and launch error capture.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/apnn.h"

namespace apnn {

char *error_buffer();                         // thread-local, 512 bytes
int fail(apnn_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// Checks the status of the launch just issued (no synchronisation).
int check_launch(const char *what);

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// bits in 1..8; +-1 only with one bit (Sec. 3.2 defines it for 1-bit operands).
int check_bits_enc(const char *who, const char *name, int bits, apnn_encoding enc);

// K (2^p - 1)(2^q - 1) must stay below 2^31 (the result type is int32, Sec. 4.1).
int check_int32_range(const char *who, int64_t K, int p, int q);

}  // namespace apnn
