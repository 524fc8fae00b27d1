// Declarations shared by the translation units of the library (not part of the C ABI).
#pragma once
#include <stdint.h>

#include <string>

struct lapis_csr;

namespace lapis {

// Records `msg` as the calling thread's last error (the text behind lapis_last_error()) and
// returns `code`.
int fail(int code, const std::string &msg);

// Bytes of the x operand (ncols values) and of the y operand (nrows values) of a product with A.
void vector_bytes(const lapis_csr *A, int64_t *x_bytes, int64_t *y_bytes);

}  // namespace lapis
