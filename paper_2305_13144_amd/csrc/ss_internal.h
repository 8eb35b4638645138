// Internal declarations shared by the library's translation units (not part of the C ABI).
#ifndef SS_INTERNAL_H
#define SS_INTERNAL_H

#include <cstddef>
#include <cstdint>
#include <exception>
#include <new>

#include "../../include/ss.h"

namespace ss {

// Records a thread-local message and returns `code` (printf-style).
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();
int verbose();   // ss_set_verbose level

// Runs the body of an entry point (a callable returning an SS_* code) so that no C++ exception crosses the C ABI:
// a failed host allocation becomes SS_ENOMEM, anything else SS_ESTATE, each with a message.
template <class Body>
int no_throw(Body&& body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(SS_ENOMEM, "host allocation failed");
    } catch (const std::exception& e) {
        return fail(SS_ESTATE, "unexpected host error: %s", e.what());
    } catch (...) {
        return fail(SS_ESTATE, "unexpected host error");
    }
}

constexpr int kMaxPos = 4096;     // positions per row (prompt + generated) the attention kernel supports
constexpr int kMaxBatch = 1024;   // rows per micro-batch the bookkeeping kernel supports

// ---- packed operand layout ---------------------------------------------------------------
// Every IEEE-half matrix that feeds an MFMA contraction (weights [N, K] and activations [rows, K]) is
// stored as 16-row strips of 16x32 blocks; a block is 64 lanes x 8 consecutive-k values, i.e. the
// register image of one mfma_f32_16x16x32_f16 operand, 1 KiB contiguous.  K is padded to 64.
inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline int padded_k(int k) { return round_up(k, 64); }
inline size_t packed_elems(int rows, int k) { return (size_t)round_up(rows, 16) * (size_t)padded_k(k); }

}  // namespace ss

#endif
